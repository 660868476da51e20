"""GPU tests of pe_stack_fwd_bwd: against the oracle (fp32) and against chained single-block calls."""
import numpy as np
import pytest
import torch

import paper_2211_00235_amd as pe
from oracle import evoformer as ev
from oracle.params import param_table
from pe_inputs import make_inputs, dims_for
from tests.gpu_util import to_dev, to_np, rel_err, tdtype

pytestmark = pytest.mark.gpu


def _stack_inputs(dims, n_blocks, seed, mask):
    table, n = param_table(dims)
    inp = make_inputs(dims, table, n, mask, seed, n_blocks=n_blocks)
    return table, n, inp


def _run_stack(dims, n_main, inp, two_streams=True, keep=False):
    dt, f32 = tdtype(dims), torch.float32
    h = pe.Handle()
    if keep:
        h.set_option(5, 1)      # PE_OPT_STACK_KEEP_CTX
    msa, pair = to_dev(inp["msa"], dt), to_dev(inp["pair"], dt)
    mm, pm = to_dev(inp["msa_mask"], f32), to_dev(inp["pair_mask"], f32)
    params = to_dev(inp["params"], f32)
    dmo, dzo = to_dev(inp["d_msa_out"], dt), to_dev(inp["d_pair_out"], dt)
    mo, zo, dmi, dzi = (torch.empty_like(t) for t in (msa, pair, msa, pair))
    dpar = torch.zeros_like(params)
    ws = torch.empty(pe.stack_workspace_bytes(0, None, n_main, dims, keep=keep), dtype=torch.uint8, device="cuda")
    sm = torch.cuda.Stream() if two_streams else torch.cuda.current_stream()
    sp = torch.cuda.Stream() if two_streams else sm
    torch.cuda.synchronize()
    pe.stack_fwd_bwd(h, 0, None, n_main, dims, None, msa, pair, None, mm, pm, params, dmo, dzo, mo, zo, None, dmi, dzi,
                     dpar, ws, sm, sp)
    torch.cuda.synchronize()
    return mo, zo, dmi, dzi, dpar


def test_stack_fp32_matches_oracle():
    """Two tiny fp32 blocks: outputs, input cotangents and all parameter gradients at 1e-4."""
    dims, mask, seed = dims_for("tiny")
    table, n, inp = _stack_inputs(dims, 2, 11, mask)
    mo, zo, dmi, dzi, dpar = _run_stack(dims, 2, inp)
    r = ev.stack_fwd_bwd(0, None, 2, dims, inp["params"], None, inp["msa"], inp["pair"], None, inp["msa_mask"],
                         inp["pair_mask"], inp["d_msa_out"], inp["d_pair_out"])
    msa_o, pair_o, _, dm, dz, g = r
    assert rel_err(to_np(mo), msa_o) < 1e-4 and rel_err(to_np(zo), pair_o) < 1e-4
    assert rel_err(to_np(dmi), dm) < 1e-4 and rel_err(to_np(dzi), dz) < 1e-4
    gg = to_np(dpar)
    for b in range(2):
        for e in table:
            k = int(np.prod(e["shape"]))
            sl = slice(b * n + e["offset"], b * n + e["offset"] + k)
            den = np.max(np.abs(g[sl]))
            if e["name"] == "row.ln_z.b":      # exactly zero gradient (a per-head constant cancels in the softmax)
                den = np.max(np.abs(g))
            assert np.max(np.abs(gg[sl] - g[sl])) / den < 1e-4, (b, e["name"])


@pytest.mark.parametrize("keep", [False, True])
@pytest.mark.parametrize("dtype", [0, 1])
def test_stack_equals_chained_blocks(dtype, keep):
    """The stack (saved block inputs + recompute, or every block's activations kept) is bit-identical
    to calling pe_block_fwd for every block and then pe_block_bwd in reverse order; this carries the
    block-level parity to any depth."""
    dims, mask, seed = dims_for("tiny")
    dims.update(dtype=dtype, s=16, r=40)
    nb = 3
    table, n, inp = _stack_inputs(dims, nb, 12, ("last_residues", 4))
    mo, zo, dmi, dzi, dpar = _run_stack(dims, nb, inp, keep=keep)
    dt, f32 = tdtype(dims), torch.float32
    h = pe.Handle()
    mm, pm = to_dev(inp["msa_mask"], f32), to_dev(inp["pair_mask"], f32)
    params = to_dev(inp["params"], f32)
    xs, zs = [to_dev(inp["msa"], dt)], [to_dev(inp["pair"], dt)]
    ws = torch.empty(pe.workspace_bytes(dims, 1), dtype=torch.uint8, device="cuda")
    # two streams, as in the stack run: a call that has the chip to itself (one stream) sums its bf16
    # parameter gradients in another order
    sm, sp = torch.cuda.Stream(), torch.cuda.Stream()
    outs = [(torch.empty_like(xs[0]), torch.empty_like(zs[0])) for _ in range(nb)]
    dm, dz = to_dev(inp["d_msa_out"], dt), to_dev(inp["d_pair_out"], dt)
    grads = [(torch.empty_like(dm), torch.empty_like(dz)) for _ in range(nb)]
    dpar2 = torch.zeros_like(params)
    torch.cuda.synchronize()
    for b in range(nb):
        xo, zo2 = outs[b]
        pe.block_fwd(h, dims, xs[b], zs[b], mm, pm, params[b * n:(b + 1) * n], xo, zo2, None, ws, sm, sp)
        xs.append(xo)
        zs.append(zo2)
    for b in reversed(range(nb)):
        dmi2, dzi2 = grads[b]
        pe.block_bwd(h, dims, xs[b], zs[b], mm, pm, params[b * n:(b + 1) * n], dm, dz, dmi2, dzi2,
                     dpar2[b * n:(b + 1) * n], None, ws, sm, sp)
        dm, dz = dmi2, dzi2
    torch.cuda.synchronize()
    assert torch.equal(mo, xs[-1]) and torch.equal(zo, zs[-1])
    assert torch.equal(dmi, dm) and torch.equal(dzi, dz) and torch.equal(dpar, dpar2)


def test_stack_bf16_error_against_oracle_by_depth(capsys):
    """bf16 main blocks (channel widths of the AF2 initial-training block, s 16, r 40) stacked 1..16 deep against
    the float64 oracle of the same stack.  The per-block tolerance is bound by the block tests and carried to
    any depth by the chained-blocks identity above; this one reports how the rounding of the bf16 residual
    stream accumulates (relative L2 error: forward outputs, input cotangents, parameter gradients) and bounds
    it by sqrt(depth) growth.  ReLU decisions are not matched here, so the backward figures include the
    O(1) gradient differences at the few pre-activations that round to the other side of zero."""
    dims, _, _ = dims_for("af2_initial")
    dims.update(s=16, r=40)
    table, n = param_table(dims)
    l2 = lambda a, b: float(np.linalg.norm(a - b) / np.linalg.norm(b))
    rows = []
    for depth in (1, 2, 4, 8, 16):
        inp = make_inputs(dims, table, n, ("last_residues", 4), 100, n_blocks=depth)
        msa_o, pair_o, _, dm, dz, g = ev.stack_fwd_bwd(0, None, depth, dims, inp["params"], None, inp["msa"], inp["pair"],
                                                       None, inp["msa_mask"], inp["pair_mask"], inp["d_msa_out"],
                                                       inp["d_pair_out"])
        mo, zo, dmi, dzi, dpar = _run_stack(dims, depth, inp)
        fwd = max(l2(to_np(mo), msa_o), l2(to_np(zo), pair_o))
        bwd = max(l2(to_np(dmi), dm), l2(to_np(dzi), dz))
        gp = l2(to_np(dpar), g)
        rows.append((depth, fwd, bwd, gp))
        assert fwd < 1e-2 * np.sqrt(depth), rows
        assert bwd < 5e-2 * np.sqrt(depth) and gp < 5e-2 * np.sqrt(depth), rows
    with capsys.disabled():
        print("\n  depth  fwd rel-L2  bwd rel-L2  dparams rel-L2")
        for r in rows:
            print("  %5d  %.3e   %.3e   %.3e" % r)


@pytest.mark.parametrize("keep", [False, True])
def test_stack_hip_graph_capture_and_replay(keep):
    """The whole stack call (here 1 extra-MSA + 3 main blocks, forward and backward, both streams) is
    captured into one HIP graph; replays, with eager work of another case in between, reproduce the
    eager result bit for bit."""
    dims_m, mask, _ = dims_for("tiny")
    dims_m.update(dtype=1, s=16, r=40)
    dims_e = dict(dims_m, s=24, c_m=16, col_global=1)
    te, ne = param_table(dims_e)
    tm, nm = param_table(dims_m)
    nb = 3
    ie = make_inputs(dims_e, te, ne, ("random_rows", 0.1), 51)
    im = make_inputs(dims_m, tm, nm, ("last_residues", 4), 52, n_blocks=nb)
    bf, f32 = torch.bfloat16, torch.float32
    par = to_dev(np.concatenate([ie["params"], im["params"]]), f32)
    ex, msa, pair = to_dev(ie["msa"], bf), to_dev(im["msa"], bf), to_dev(im["pair"], bf)
    exm, mm, pm = to_dev(ie["msa_mask"], f32), to_dev(im["msa_mask"], f32), to_dev(im["pair_mask"], f32)
    dmo, dzo = to_dev(im["d_msa_out"], bf), to_dev(im["d_pair_out"], bf)
    mo, zo, dex, dmi, dzi = (torch.empty_like(t) for t in (msa, pair, ex, msa, pair))
    dpar = torch.zeros_like(par)
    h = pe.Handle()
    if keep:
        h.set_option(5, 1)      # PE_OPT_STACK_KEEP_CTX
    ws = torch.empty(pe.stack_workspace_bytes(1, dims_e, nb, dims_m, keep=keep), dtype=torch.uint8, device="cuda")
    sm, sp = torch.cuda.Stream(), torch.cuda.Stream()
    outs = (mo, zo, dex, dmi, dzi, dpar)

    def call():
        pe.stack_fwd_bwd(h, 1, dims_e, nb, dims_m, ex, msa, pair, exm, mm, pm, par, dmo, dzo, mo, zo, dex, dmi, dzi,
                         dpar, ws, sm, sp)
    torch.cuda.synchronize()
    call()
    torch.cuda.synchronize()
    ref = [t.clone() for t in outs]
    dpar.zero_()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=sm):
        call()
    other = torch.randn(1 << 20, device="cuda")
    for rep in range(3):
        for t in outs:
            t.zero_()
        ws.zero_()
        other = other * 1.0001 + 1.0     # unrelated eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (t, r) in enumerate(zip(outs, ref)):
            assert torch.equal(t, r), (rep, i)


def test_trunk_full_size_equals_chained_blocks():
    """The trunk the bench times (4 extra-MSA blocks at s 1024 then 48 main blocks at s 128, r 256, bf16, every
    block's activations kept: 69 GiB of workspace, offsets beyond 32 bits) is bit-identical to chaining
    pe_block_fwd over the 52 blocks and pe_block_bwd (recompute) back over them.  With the block-level parity
    at these shapes this carries the oracle comparison to the full-size trunk, which the float64 oracle
    itself cannot run in test time."""
    de, me, _ = dims_for("extra_msa")
    dm, mmk, _ = dims_for("af2_initial")
    ne, nm = 4, 48
    te, n_e = param_table(de)
    tm, n_m = param_table(dm)
    ie = make_inputs(de, te, n_e, me, 4, n_blocks=ne)
    im = make_inputs(dm, tm, n_m, mmk, 5, n_blocks=nm)
    bf, f32 = torch.bfloat16, torch.float32
    ex, msa, pair = to_dev(ie["msa"], bf), to_dev(im["msa"], bf), to_dev(im["pair"], bf)
    exm, mm, pm = to_dev(ie["msa_mask"], f32), to_dev(im["msa_mask"], f32), to_dev(im["pair_mask"], f32)
    par = torch.cat([to_dev(ie["params"], f32), to_dev(im["params"], f32)])
    dmo, dzo = to_dev(im["d_msa_out"], bf), to_dev(im["d_pair_out"], bf)
    mo, zo, dex, dmi, dzi = (torch.empty_like(t) for t in (msa, pair, ex, msa, pair))
    dpar = torch.zeros_like(par)
    h = pe.Handle()
    h.set_option(5, 1)      # PE_OPT_STACK_KEEP_CTX
    ws = torch.empty(pe.stack_workspace_bytes(ne, de, nm, dm, keep=True), dtype=torch.uint8, device="cuda")
    assert ws.numel() > (1 << 32)
    sm, sp = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    pe.stack_fwd_bwd(h, ne, de, nm, dm, ex, msa, pair, exm, mm, pm, par, dmo, dzo, mo, zo, dex, dmi, dzi, dpar, ws, sm, sp)
    torch.cuda.synchronize()
    del ws
    torch.cuda.empty_cache()

    h2 = pe.Handle()
    wsb = torch.empty(max(pe.workspace_bytes(de, 1), pe.workspace_bytes(dm, 1)), dtype=torch.uint8, device="cuda")
    off = lambda b: b * n_e if b < ne else ne * n_e + (b - ne) * n_m
    xs_e, xs_m, zs = [ex], [msa], [pair]
    for b in range(ne + nm):
        is_e = b < ne
        d_, x, mk = (de, xs_e[-1], exm) if is_e else (dm, xs_m[-1], mm)
        n_ = n_e if is_e else n_m
        xo, z2 = torch.empty_like(x), torch.empty_like(pair)
        pe.block_fwd(h2, d_, x, zs[-1], mk, pm, par[off(b):off(b) + n_], xo, z2, None, wsb, sm, sp)
        (xs_e if is_e else xs_m).append(xo)
        zs.append(z2)
    torch.cuda.synchronize()
    assert torch.equal(mo, xs_m[-1]) and torch.equal(zo, zs[-1])
    dpar2 = torch.zeros_like(par)
    g_m, g_e, g_z = dmo, torch.zeros_like(ex), dzo
    for b in reversed(range(ne + nm)):
        is_e = b < ne
        d_, mk, n_ = (de, exm, n_e) if is_e else (dm, mm, n_m)
        x = xs_e[b] if is_e else xs_m[b - ne]
        gx_in = g_e if is_e else g_m
        gx, gz = torch.empty_like(x), torch.empty_like(pair)
        pe.block_bwd(h2, d_, x, zs[b], mk, pm, par[off(b):off(b) + n_], gx_in, g_z, gx, gz,
                     dpar2[off(b):off(b) + n_], None, wsb, sm, sp)
        if is_e:
            g_e = gx
        else:
            g_m = gx
        g_z = gz
    torch.cuda.synchronize()
    assert torch.equal(dmi, g_m) and torch.equal(dex, g_e) and torch.equal(dzi, g_z)
    assert torch.equal(dpar, dpar2)
    assert bool(torch.isfinite(dpar).all()) and bool(torch.isfinite(zo.float()).all())


def test_stack_argument_errors():
    dims, mask, seed = dims_for("tiny")
    table, n, inp = _stack_inputs(dims, 1, 1, mask)
    h = pe.Handle()
    t = to_dev(inp["pair"], torch.float32)
    small = torch.empty(1024, dtype=torch.uint8, device="cuda")
    with pytest.raises(pe.PEError, match="workspace too small"):
        m = to_dev(inp["msa"], torch.float32)
        pe.stack_fwd_bwd(h, 0, None, 1, dims, None, m, t, None, to_dev(inp["msa_mask"], torch.float32),
                         to_dev(inp["pair_mask"], torch.float32), to_dev(inp["params"], torch.float32), m, t,
                         torch.empty_like(m), torch.empty_like(t), None, torch.empty_like(m), torch.empty_like(t),
                         torch.zeros(n, device="cuda"), small)


@pytest.mark.parametrize("n_extra,n_main", [(1, 1), (2, 2), (3, 1)])
def test_stack_extra_then_main_fp32_matches_oracle(n_extra, n_main):
    """Extra-MSA blocks (global column attention, their own s and c_m) followed by main blocks: the pair
    representation chains through all of them, the extra-MSA representation is dropped.  Odd and even counts
    of extra blocks (the cotangent of the dropped representation starts as zero in the ping-pong slot that the
    last extra block does not write).  Every output, input cotangent and parameter-gradient entry at 1e-4."""
    dims_m, mask, seed = dims_for("tiny")
    dims_e = dict(dims_m, s=24, c_m=16, col_global=1)
    te, ne = param_table(dims_e)
    tm, nm = param_table(dims_m)
    ie = make_inputs(dims_e, te, ne, ("random_rows", 0.1), 41, n_blocks=n_extra)
    im = make_inputs(dims_m, tm, nm, mask, 42, n_blocks=n_main)
    params = np.concatenate([ie["params"], im["params"]])
    f32 = torch.float32
    h = pe.Handle()
    dev = lambda a: to_dev(a, f32)
    ex, msa, pair = dev(ie["msa"]), dev(im["msa"]), dev(im["pair"])
    exm, mm, pm = dev(ie["msa_mask"]), dev(im["msa_mask"]), dev(im["pair_mask"])
    par = dev(params)
    dmo, dzo = dev(im["d_msa_out"]), dev(im["d_pair_out"])
    mo, zo, dex, dmi, dzi = (torch.empty_like(t) for t in (msa, pair, ex, msa, pair))
    dpar = torch.zeros_like(par)
    ws = torch.empty(pe.stack_workspace_bytes(n_extra, dims_e, n_main, dims_m), dtype=torch.uint8, device="cuda")
    ws.fill_(0x7F)     # stale bytes (large finite values) wherever the call reads something it has not written
    sm, sp = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    pe.stack_fwd_bwd(h, n_extra, dims_e, n_main, dims_m, ex, msa, pair, exm, mm, pm, par, dmo, dzo, mo, zo, dex, dmi,
                     dzi, dpar, ws, sm, sp)
    torch.cuda.synchronize()
    r = ev.stack_fwd_bwd(n_extra, dims_e, n_main, dims_m, params, ie["msa"], im["msa"], im["pair"], ie["msa_mask"],
                         im["msa_mask"], im["pair_mask"], im["d_msa_out"], im["d_pair_out"])
    msa_o, pair_o, de, dm, dz, g = r
    for got, ref in ((mo, msa_o), (zo, pair_o), (dex, de), (dmi, dm), (dzi, dz)):
        assert rel_err(to_np(got), ref) < 1e-4
    gg = to_np(dpar)
    blocks = [(b * ne, te) for b in range(n_extra)] + [(n_extra * ne + b * nm, tm) for b in range(n_main)]
    for off, table in blocks:
        for e in table:
            k = int(np.prod(e["shape"]))
            sl = slice(off + e["offset"], off + e["offset"] + k)
            den = np.max(np.abs(g[sl]))
            if e["name"] == "row.ln_z.b":      # exactly zero gradient (a per-head constant cancels in the softmax)
                den = np.max(np.abs(g))
            assert np.max(np.abs(gg[sl] - g[sl])) / den < 1e-4, (off, e["name"])


def test_stack_needs_both_branches():
    """A block with one branch switched off leaves an output unwritten that the next block would read."""
    dims, mask, seed = dims_for("tiny")
    table, n, inp = _stack_inputs(dims, 1, 1, mask)
    h = pe.Handle()
    h.set_option(1, 1)
    f32 = torch.float32
    m, t = to_dev(inp["msa"], f32), to_dev(inp["pair"], f32)
    ws = torch.empty(pe.stack_workspace_bytes(0, None, 1, dims), dtype=torch.uint8, device="cuda")
    with pytest.raises(pe.PEError, match="both branches"):
        pe.stack_fwd_bwd(h, 0, None, 1, dims, None, m, t, None, to_dev(inp["msa_mask"], f32),
                         to_dev(inp["pair_mask"], f32), to_dev(inp["params"], f32), m.clone(), t.clone(),
                         torch.empty_like(m), torch.empty_like(t), None, torch.empty_like(m), torch.empty_like(t),
                         torch.zeros(n, device="cuda"), ws)


@pytest.mark.parametrize("dtype", [0, 1])
def test_stack_cross_block_overlap_is_bit_identical(dtype):
    """Trunk-level scheduling: with every block's activations kept, the next block's row-attention LayerNorm and
    q / k / v / gate projection (and its MSA-side weight preparation) are enqueued on stream_msa before the current
    block's outer product mean waits for the pair branch.  2 extra-MSA + 3 main blocks (the overlap crosses the
    extra -> main boundary, where the next block reads the caller's MSA input): every output, input cotangent and
    parameter gradient is bit-identical with the overlap switched off (PE_OPT_STACK_OVERLAP = 0)."""
    dims_m, mask, seed = dims_for("tiny")
    dims_m.update(dtype=dtype, s=16, r=40)
    dims_e = dict(dims_m, s=24, c_m=16, col_global=1)
    n_extra, n_main = 2, 3
    te, ne = param_table(dims_e)
    tm, nm = param_table(dims_m)
    ie = make_inputs(dims_e, te, ne, ("random_rows", 0.1), 71, n_blocks=n_extra)
    im = make_inputs(dims_m, tm, nm, ("last_residues", 4), 72, n_blocks=n_main)
    dt, f32 = tdtype(dims_m), torch.float32
    ex, msa, pair = to_dev(ie["msa"], dt), to_dev(im["msa"], dt), to_dev(im["pair"], dt)
    exm, mm, pm = to_dev(ie["msa_mask"], f32), to_dev(im["msa_mask"], f32), to_dev(im["pair_mask"], f32)
    par = to_dev(np.concatenate([ie["params"], im["params"]]), f32)
    dmo, dzo = to_dev(im["d_msa_out"], dt), to_dev(im["d_pair_out"], dt)
    results = []
    for overlap in (1, 0):
        h = pe.Handle()
        h.set_option(5, 1)          # PE_OPT_STACK_KEEP_CTX
        h.set_option(6, overlap)    # PE_OPT_STACK_OVERLAP
        outs = [torch.empty_like(t) for t in (msa, pair, ex, msa, pair)]
        dpar = torch.zeros_like(par)
        ws = torch.empty(pe.stack_workspace_bytes(n_extra, dims_e, n_main, dims_m, keep=True), dtype=torch.uint8,
                         device="cuda")
        ws.fill_(0x7F)
        sm, sp = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        pe.stack_fwd_bwd(h, n_extra, dims_e, n_main, dims_m, ex, msa, pair, exm, mm, pm, par, dmo, dzo, outs[0], outs[1],
                         outs[2], outs[3], outs[4], dpar, ws, sm, sp)
        torch.cuda.synchronize()
        results.append(outs + [dpar])
    for a, b in zip(*results):
        assert torch.isfinite(a.float()).all()
        assert torch.equal(a, b)
