#!/usr/bin/env python3
"""Benchmark: one Parallel Evoformer block forward + backward on one MI355X.

A "step" is one pass of the whole hot path (pe_block_fwd with saved ctx, then
pe_block_fwd's ctx consumed by pe_block_bwd) over one synthetic AlphaFold2
initial-training batch (s=128, r=256, c_m=256, c_z=128, bf16 storage, fp32
accumulate), MSA branch and pair branch on two HIP streams.  Inputs are
resident in HBM before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
PAPER_MS_PER_LAYER = 32.47    # paper Table 5, PPFold DAP=1 BP=1, 1x A100 40G, fp16, same shape


def block_fwd_flops(d):
    """Algorithmic forward flops (2*M*N*K per contraction, masked positions counted dense)."""
    s, r, cm, cz = d["s"], d["r"], d["c_m"], d["c_z"]
    Mm, Mz = s * r, r * r
    Hm, dm, Hp, dp = d["h_msa"], d["d_msa"], d["h_pair"], d["d_pair"]
    ct, co, n = d["c_tri"], d["c_opm"], d["n_trans"]
    f = 0.0
    f += 2 * Mm * cm * 5 * Hm * dm + 2 * Mz * cz * Hm + 4 * s * Hm * r * r * dm          # row attention
    f += 2 * Mm * cm * 5 * Hm * dm + 4 * r * Hm * s * s * dm                             # column attention
    f += 4 * Mm * cm * n * cm                                                            # MSA transition
    f += 2 * Mm * cm * 2 * co + 2 * (r * co) ** 2 * s + 2 * Mz * co * co * cz            # outer product mean
    f += 2 * (2 * Mz * cz * (4 * ct + cz) + 2 * Mz * ct * cz + 2 * r ** 3 * ct)          # triangle multiplication x2
    f += 2 * (2 * Mz * cz * 5 * Hp * dp + 2 * Mz * cz * Hp + 4 * r * Hp * r * r * dp)    # triangle attention x2
    f += 4 * Mz * cz * n * cz                                                            # pair transition
    return f


def bench_trunk(args, torch, pe):
    """Config 5: 4 extra-MSA blocks then 48 main blocks, per-block recompute, two streams."""
    from pe_inputs import dims_for, make_inputs
    from paper_2211_00235_amd.harness import to_dev
    de, me, _ = dims_for("extra_msa")
    dm, mmk, _ = dims_for("af2_initial")
    ne, nm = 4, 48
    te, tm = pe.param_table(de), pe.param_table(dm)
    ie = make_inputs(de, te, pe.param_count(de), me, 4, n_blocks=ne)
    im = make_inputs(dm, tm, pe.param_count(dm), mmk, 5, n_blocks=nm)
    bf, f32 = torch.bfloat16, torch.float32
    ex, msa, pair = to_dev(ie["msa"], bf), to_dev(im["msa"], bf), to_dev(im["pair"], bf)
    exm, mm, pm = to_dev(ie["msa_mask"], f32), to_dev(im["msa_mask"], f32), to_dev(im["pair_mask"], f32)
    par = torch.cat([to_dev(ie["params"], f32), to_dev(im["params"], f32)])
    dmo, dzo = to_dev(im["d_msa_out"], bf), to_dev(im["d_pair_out"], bf)
    mo, zo, dex, dmi, dzi = (torch.empty_like(t) for t in (msa, pair, ex, msa, pair))
    dpar = torch.zeros_like(par)
    keep = not args.recompute
    ws = torch.empty(pe.stack_workspace_bytes(ne, de, nm, dm, keep=keep), dtype=torch.uint8, device="cuda")
    h = pe.Handle()
    if keep:
        h.set_option(5, 1)      # PE_OPT_STACK_KEEP_CTX: 288 GB hold every block's activations
    if args.no_overlap:
        h.set_option(6, 0)      # PE_OPT_STACK_OVERLAP off: no kernels of the next block before the current one's join
    sm, sp = torch.cuda.Stream(), torch.cuda.Stream()

    def eager():
        pe.stack_fwd_bwd(h, ne, de, nm, dm, ex, msa, pair, exm, mm, pm, par, dmo, dzo, mo, zo, dex, dmi, dzi, dpar,
                         ws, sm, sp)
    step = eager
    if args.graph:              # the whole trunk (about 9000 launches on two streams) as one HIP graph
        eager()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=sm):
            eager()

        def step():
            with torch.cuda.stream(sm):
                graph.replay()
    steps, warm = max(1, min(args.steps, 5)), max(1, min(args.warmup, 2))
    for _ in range(warm):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    flops = 3.0 * (ne * block_fwd_flops(de) + nm * block_fwd_flops(dm))
    cpu = None
    if not args.no_cpu_baseline:
        # bounded sample: one block of each kind through the float64 oracle, scaled to the trunk's depth
        from oracle import evoformer as ev      # cpu_baseline leg only
        t_kind = []
        for d_, i_, n_ in ((de, ie, pe.param_count(de)), (dm, im, pe.param_count(dm))):
            t = time.perf_counter()
            dmo_ = i_["d_msa_out"] if d_ is dm else np.zeros_like(i_["msa"])
            ev.block_fwd_bwd(d_, i_["params"][:n_], i_["msa"], im["pair"], i_["msa_mask"], im["pair_mask"], dmo_,
                             im["d_pair_out"])
            t_kind.append((time.perf_counter() - t) * 1e3)
        cpu = {"value": ne * t_kind[0] + nm * t_kind[1], "unit": "ms", "cores": os.cpu_count(), "kind": "oracle",
               "sample": "one extra-MSA block (%.0f ms) and one main block (%.0f ms) fwd+bwd in float64 numpy, "
                         "scaled to 4 + 48 blocks (no recompute)" % (t_kind[0], t_kind[1])}
    print(json.dumps({
        "metric": "Parallel Evoformer trunk (4 extra + 48 main blocks) fwd+bwd ms", "value": ms, "unit": "ms",
        "n_gpus": 1, "steps": steps, "warmup": warm, "ms_per_step": ms, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "trunk", "n_extra": ne, "n_main": nm, "streams": 2,
                   "launch": "hip graph replay" if args.graph else "eager",
                   "cross_block_overlap": bool(keep and not args.no_overlap),
                   "recompute": "none (every block's activations kept)" if keep else "per block",
                   "workspace_gib": round(ws.numel() / 2 ** 30, 1)},
        "counted_tflops": flops / (ms * 1e-3) / 1e12,
        "bf16_mfma_peak_frac": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "finite_outputs": bool(torch.isfinite(zo.float()).all().item() and torch.isfinite(dpar).all().item()),
        "cpu_baseline": cpu}))


def kernel_symbol(name, dims):
    """Launch labels carry the kernel as written at the launch site, e.g. "(attn_fwd_kernel<T, true>)"; bring them to
    the form of the kernel symbol in a rocprofv3 trace ("attn_fwd_kernel<bf16,true>")."""
    t = "bf16" if dims["dtype"] == 1 else "f32"
    name = name.strip("()").replace(" ", "")
    return name.replace("<T,", "<%s," % t).replace("<T>", "<%s>" % t)


def profiled_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary of this workload
    (FETCH_SIZE and WRITE_SIZE runs, scaled by what a plain copy reads on the same counters).  None
    when there is no summary for the workload or it does not list exactly this kernel: a summary
    taken before a kernel was renamed or replaced yields no figure instead of a stale one."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles",
                        "block_fwd_bwd_%s_hbm_traffic.md" % workload)
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic:" and f[1] == kernel:
                return float(f[2])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="af2_initial")
    ap.add_argument("--variant", type=int, default=0, choices=[0, 1, 2],
                    help="block ordering of Figure 1: 0 Parallel Evoformer (the headline), 1 AlphaFold2, 2 Multimer")
    ap.add_argument("--recompute", action="store_true",
                    help="trunk workload: save block inputs only and recompute each block's forward in the backward "
                         "pass (the paper's memory-saving setting) instead of keeping every block's activations")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step (both streams) into a HIP graph once and time graph replays")
    ap.add_argument("--no-overlap", action="store_true",
                    help="trunk workload: do not start the next block's row-attention LayerNorm and projections "
                         "before the current block's pair branch has finished")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--detail", action="store_true", help="also print the per-launch-label timing table to stderr")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run three 256 MiB device-to-device copies (known traffic: the scale of the "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE counters is read off them)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the one-GPU share of the path only (two HIP streams on one "
              "MI355X); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2211_00235_amd as pe
    from pe_inputs import dims_for, make_inputs
    from paper_2211_00235_amd.harness import BlockRun     # argument marshalling helper (no oracle import)

    pe.lib()                                  # fails loudly when the HIP library is not built
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    if args.copy_calibration:
        x = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda")
        y = torch.empty_like(x)
        for _ in range(3):
            y.copy_(x)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_each_way": 256 << 20, "copies": 3}))
        return
    if args.workload == "trunk":
        return bench_trunk(args, torch, pe)
    dims, mask, seed = dims_for(args.workload)
    dims["variant"] = args.variant
    table = pe.param_table(dims)
    inp = make_inputs(dims, table, pe.param_count(dims), mask, seed)
    run = BlockRun(dims, inp, two_streams=True)

    def step():
        run.fwd(use_ctx=True)
        run.bwd(use_ctx=True)

    eager_step = step
    if args.graph:
        eager_step()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=run.sm):
            eager_step()

        def step():
            with torch.cuda.stream(run.sm):
                graph.replay()
    for _ in range(args.warmup):
        step()
    # one event per step boundary on the MSA stream (both streams are joined at every return, so
    # the event after step k completes when step k has); the headline is the host-clocked mean
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record(run.sm)
    for i in range(args.steps):
        step()
        marks[i + 1].record(run.sm)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    ms_median = per_step[len(per_step) // 2]

    # ---- branch overlap (a few untimed-in-the-headline iterations each) ----
    def timed(n, fn):
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(n):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / n
    nrep = max(3, min(10, args.steps))
    t_msa = t_pair = overlap = None
    if args.variant == 0:       # only the Parallel block has two independent branches to time alone
        run.h.set_option(1, 1)
        t_msa = timed(nrep, eager_step)
        run.h.set_option(1, 2)
        t_pair = timed(nrep, eager_step)
        run.h.set_option(1, 3)
        overlap = (t_msa + t_pair - ms) / min(t_msa, t_pair)
    one = BlockRun(dims, inp, two_streams=False)
    t_serial = timed(nrep, lambda: (one.fwd(), one.bwd()))

    # ---- per-kernel timing with HIP events on the launching stream ----
    one.h.set_option(3, 1)
    for _ in range(3):
        one.fwd()
        one.bwd()
    ent = one.h.timing_collect()
    one.h.set_option(3, 0)
    if args.detail:
        for e in sorted(ent, key=lambda e: -e["total_ms"]):
            print("%-22s %-44s n=%3d  %8.1f us/launch  %7.1f TFLOP/s  %7.1f GB/s" % (
                e["name"], e["kernel"], e["launches"] // 3, 1e3 * e["total_ms"] / e["launches"],
                e["flops"] / (e["total_ms"] * 1e-3) / 1e12, e["bytes"] / (e["total_ms"] * 1e-3) / 1e9), file=sys.stderr)
    for e in ent:
        e["kernel"] = kernel_symbol(e["kernel"], dims)
    by_kernel = {}
    for e in ent:
        k = by_kernel.setdefault(e["kernel"], dict(ms=0.0, launches=0, flops=0.0, bytes=0.0))
        k["ms"] += e["total_ms"] / 3
        k["launches"] += e["launches"] // 3
        k["flops"] += e["flops"] / 3
        k["bytes"] += e["bytes"] / 3
    # the roofline entry is measured in the timed configuration itself (two streams: kernels of
    # the two branches share the chip, as they do in the timed region and in a rocprofv3 trace of
    # this command); kernels_ms_per_step above is the one-stream view of every kernel alone
    run.h.set_option(3, 1)
    for _ in range(5):
        eager_step()
    ent2 = run.h.timing_collect()
    run.h.set_option(3, 0)
    for e in ent2:
        e["kernel"] = kernel_symbol(e["kernel"], dims)
    if args.detail:
        alone = {(e["name"], e["kernel"]): e["total_ms"] / max(e["launches"], 1) for e in ent}
        # a launch that takes another kernel when it runs alone (parameter gradients): match by label only
        alone_by_name = {}
        for e in ent:
            a = alone_by_name.setdefault(e["name"], [0.0, 0])
            a[0] += e["total_ms"]
            a[1] += e["launches"]
        print("-- two streams (us/launch, ratio to the same launch alone) --", file=sys.stderr)
        for e in sorted(ent2, key=lambda e: -e["total_ms"])[:40]:
            us = 1e3 * e["total_ms"] / e["launches"]
            a = 1e3 * alone.get((e["name"], e["kernel"]), 0.0)
            if not a and e["name"] in alone_by_name:
                a = 1e3 * alone_by_name[e["name"]][0] / max(alone_by_name[e["name"]][1], 1)
            print("%-22s %-44s n=%3d  %8.1f us/launch  x%.2f" % (e["name"], e["kernel"], e["launches"] // 5, us,
                                                                   us / a if a else 0.0), file=sys.stderr)
    two = {}
    for e in ent2:
        k = two.setdefault(e["kernel"], dict(ms=0.0, launches=0, flops=0.0, bytes=0.0))
        k["ms"] += e["total_ms"] / 5
        k["launches"] += e["launches"] // 5
        k["flops"] += e["flops"] / 5
        k["bytes"] += e["bytes"] / 5
    # The roofline entry is ONE kernel symbol (for the GEMMs: one instantiation, feature mask included): the
    # one with the largest total time in the timed configuration (two streams).
    dom_name = max(two, key=lambda k: two[k]["ms"])
    dom = two[dom_name]
    # roofline model: the kernel's algorithmic intensity against the ridge (peak flops / peak bandwidth)
    # decides which roof bounds it; a contraction below the ridge is bound by HBM, not by the MFMA peak
    intensity = dom["flops"] / max(dom["bytes"], 1.0)
    ridge = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    tflops = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
    gbs = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
    if dom["flops"] > 0 and intensity >= ridge:
        roof = dict(bound="mfma", achieved=tflops, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s", frac=tflops / PEAK_BF16_TFLOPS)
    else:
        roof = dict(bound="hbm", achieved=gbs, peak=PEAK_HBM_GBS, unit="GB/s", frac=gbs / PEAK_HBM_GBS)
    roof["traffic"] = profiled_traffic(dom_name, args.workload)
    roof.update(kernel=dom_name, launches_per_step=dom["launches"],
                algorithmic_bytes_per_launch=dom["bytes"] / max(dom["launches"], 1),
                algorithmic_flops_per_launch=dom["flops"] / max(dom["launches"], 1),
                flop_per_byte=intensity, ridge_flop_per_byte=ridge,
                two_streams={"avg_launch_us": 1e3 * dom["ms"] / max(dom["launches"], 1), "ms_per_step": dom["ms"],
                             "gbs": gbs, "tflops": tflops, "mfma_peak_frac": tflops / PEAK_BF16_TFLOPS})
    # the same launches (matched by launch label: a call that has the chip to itself may take another kernel for
    # them) with both branches on one stream, i.e. every kernel alone on the chip
    labels = {e["name"] for e in ent2 if e["kernel"] == dom_name}
    a_ms = sum(e["total_ms"] for e in ent if e["name"] in labels) / 3
    a_n = sum(e["launches"] for e in ent if e["name"] in labels) // 3
    if a_n:
        roof["one_stream"] = {"avg_launch_us": 1e3 * a_ms / a_n, "ms_per_step": a_ms, "launches_per_step": a_n,
                              "gbs": dom["bytes"] / max(dom["launches"], 1) * a_n / (a_ms * 1e-3) / 1e9,
                              "kernels": sorted({e["kernel"] for e in ent if e["name"] in labels})}
    kernels = {k: dict(ms=round(v["ms"], 4), launches=v["launches"],
                       tflops=round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 2) if v["ms"] > 0 else 0.0,
                       gbs=round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["ms"] > 0 else 0.0)
               for k, v in sorted(by_kernel.items(), key=lambda kv: -kv[1]["ms"])}
    kernels2 = {k: dict(ms=round(v["ms"], 4), launches=v["launches"],
                        tflops=round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 2) if v["ms"] > 0 else 0.0,
                        gbs=round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["ms"] > 0 else 0.0)
                for k, v in sorted(two.items(), key=lambda kv: -kv[1]["ms"])}

    flops = 3.0 * block_fwd_flops(dims)
    out = {
        "metric": "Parallel Evoformer block fwd+bwd ms (s=%d,r=%d) + %% bf16 MFMA peak" % (dims["s"], dims["r"]),
        "value": ms, "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "ms_median": ms_median, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": ms / PAPER_MS_PER_LAYER if args.workload == "af2_initial" and args.variant == 0 else None,
        "baseline_note": "paper Table 5: 32.47 ms per Evoformer layer fwd+bwd, PPFold on 1x A100 40G, fp16, at the "
                         "af2_initial shape (other hardware: context, not the target)",
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "s": dims["s"], "r": dims["r"], "c_m": dims["c_m"], "c_z": dims["c_z"],
                   "batch": 1, "streams": 2, "activation_ctx": "saved", "launch": "hip graph replay" if args.graph else "eager",
                   "block_ordering": ["parallel", "alphafold2", "multimer"][args.variant]},
        "samples_per_s": 1e3 / ms,
        "block_tflops": flops / (ms * 1e-3) / 1e12,
        "bf16_mfma_peak_frac": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "overlap": {"t_msa_only_ms": t_msa, "t_pair_only_ms": t_pair, "t_two_streams_ms": ms,
                    "t_one_stream_ms": t_serial, "ratio": overlap},
        "roofline": roof,
        "kernels_two_streams_ms_per_step": kernels2,
        "kernels_one_stream_ms_per_step": kernels,
    }

    if args.workload == "extra_msa_finetune":
        out["cpu_baseline"] = None      # 6e9 float64 logits per attention: beyond the host's memory
    elif not args.no_cpu_baseline:
        from oracle import evoformer as ev      # cpu_baseline leg only
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count()])
        except Exception:
            cores = os.cpu_count()
        t = time.perf_counter()
        ev.block_fwd_bwd(dims, inp["params"], inp["msa"], inp["pair"], inp["msa_mask"], inp["pair_mask"],
                         inp["d_msa_out"], inp["d_pair_out"])
        cpu_ms = (time.perf_counter() - t) * 1e3
        model = ""
        try:
            with open("/proc/cpuinfo") as f:
                model = next((l.split(":", 1)[1].strip() for l in f if l.startswith("model name")), "")
        except OSError:
            pass
        out["cpu_baseline"] = {"value": cpu_ms, "unit": "ms", "cores": int(cores), "kind": "oracle",
                               "sample": "one full fwd+bwd of the same %s block, float64 numpy" % args.workload,
                               "os_cpu_count": os.cpu_count(), "blas_threads": int(cores), "cpu_model": model}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
