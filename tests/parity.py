"""Parity check of the HIP path against the float64 oracle for one seeded case.

ReLU decisions.  The transition's ReLU turns a floating-point pre-activation into an
on/off decision.  A pre-activation whose magnitude is below the implementation's own
rounding error of it (bf16 operands in the contraction, bf16 residual stream upstream)
has no unique decision at that precision: both are correct, and a flipped decision
changes the gradient by O(1) at that element.  The check therefore (1) requires the HIP
path's decisions to equal sign(a_oracle) wherever |a_oracle| exceeds a band, (2) takes the
HIP path's decision inside the band as one of the valid choices, and (3) compares every
output and gradient with the oracle evaluated under exactly those decisions.  The band
and the fraction of elements inside it are reported and bounded.
"""
import numpy as np

import paper_2211_00235_amd as pe
from oracle import evoformer as ev
from tests.gpu_util import BlockRun, to_np, rel_err, param_errors

TOL = {pe.PE_F32: 1e-4, pe.PE_BF16: 2e-2}
# band for ambiguous ReLU decisions, as a fraction of the rms pre-activation
BAND = {pe.PE_F32: 2e-5, pe.PE_BF16: 6e-2}


def relu_decisions(dims, run, inter):
    """Merge oracle decisions (outside the band) with the HIP path's (inside)."""
    out, stats = {}, {}
    for key, name in (("mtrans", "mtrans.h"), ("ptrans", "ptrans.h")):
        a = inter[key + "_pre"]
        h = run.ctx_entry(name).reshape(a.shape)
        band = BAND[dims["dtype"]] * np.sqrt(np.mean(a * a))
        inside = np.abs(a) <= band
        gpu_on = h > 0
        wrong = (~inside) & (gpu_on != (a > 0))
        stats[key] = dict(frac_inside=float(inside.mean()), wrong_outside=int(wrong.sum()),
                          flips_inside=int((inside & (gpu_on != (a > 0))).sum()))
        out[key] = np.where(inside, gpu_on, a > 0)
    return out, stats


def check_case(dims, table, inp, two_streams=True, use_ctx=True, verbose=False):
    tol = TOL[dims["dtype"]]
    args = (dims, inp["params"], inp["msa"], inp["pair"], inp["msa_mask"], inp["pair_mask"])
    _, _, _, inter0 = ev.block_fwd(*args, want_cache=False)
    run = BlockRun(dims, inp, two_streams=two_streams)
    run.fwd(use_ctx=True)
    run.sync()
    on, stats = relu_decisions(dims, run, inter0)
    for k, st in stats.items():
        assert st["wrong_outside"] == 0, (k, st)
        assert st["frac_inside"] < 0.08, (k, st)
    m, z, cache, inter = ev.block_fwd(*args, relu_on=on)
    dm, dz, g, _ = ev.block_bwd(dims, cache, inp["d_msa_out"], inp["d_pair_out"])
    errs = {}
    # saved residual-stream values; with the outer product mean in front of the pair stack (orderings
    # (a) and (b) of Figure 1) z0 = pair input + outer product mean is saved and z5 is the output itself
    keys = ("m1", "m2", "m3", "z1", "z2", "z3", "z4") + (("z0",) if dims.get("variant", 0) else ("z5",))
    for k in keys:
        errs["ctx." + k] = rel_err(run.ctx_entry(k).reshape(inter[k].shape), inter[k])
    errs["msa_out"] = rel_err(to_np(run.msa_out), m)
    errs["pair_out"] = rel_err(to_np(run.pair_out), z)
    if not use_ctx:
        run.ctx.zero_()
        run.sync()
    run.bwd(use_ctx=use_ctx)
    run.sync()
    errs["d_msa_in"] = rel_err(to_np(run.d_msa_in), dm)
    errs["d_pair_in"] = rel_err(to_np(run.d_pair_in), dz)
    perr = param_errors(to_np(run.d_params), g, table)
    errs.update({"d_params." + k: v for k, v in perr.items()})
    worst = max(errs, key=errs.get)
    if verbose:
        for k, v in errs.items():
            print("  %-26s %.3e" % (k, v))
        print("  relu:", stats)
    return errs, worst, tol, stats
