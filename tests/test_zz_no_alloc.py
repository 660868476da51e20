"""pe_block_fwd_static (the entry point for callers that cannot allocate device memory) against
pe_block_fwd on the same inputs, through the C ABI: two calls in a row on the same handle, the second
with a smaller input, then a bf16 case; outputs must be bit-identical (same kernels, same order)."""
import pytest
import torch

import paper_2211_00235_amd as pe
from oracle.params import param_table
from pe_inputs import make_inputs, dims_for
from tests.gpu_util import BlockRun

pytestmark = pytest.mark.gpu


def _inputs(seed, **over):
    dims, mask, _ = dims_for("tiny")
    dims.update(over)
    table, n = param_table(dims)
    return dims, make_inputs(dims, table, n, mask, seed)


def test_static_scratch_forward_matches_workspace_forward():
    cases = [_inputs(51, s=24, r=48), _inputs(52), _inputs(53, s=16, r=64, c_m=64, c_z=32, dtype=1)]
    limit = pe.static_scratch_bytes()
    for dims, _ in cases:
        assert pe.workspace_bytes(dims, 1) <= limit
    assert pe.workspace_bytes(cases[0][0], 1) > pe.workspace_bytes(cases[1][0], 1)   # second call is the smaller one
    runs = [BlockRun(dims, inp) for dims, inp in cases]
    for run in runs:                       # reference: the existing entry point, caller's workspace
        run.fwd(use_ctx=False)
    torch.cuda.synchronize()
    refs = [(run.msa_out.clone(), run.pair_out.clone()) for run in runs]
    h = runs[0].h
    sm, sp = runs[0].sm, runs[0].sp
    for run in runs:
        run.msa_out.zero_()
        run.pair_out.zero_()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for run in runs:                       # back to back on the same streams: ordered, no race on the shared array
        pe.block_fwd_static(h, run.dims, run.msa, run.pair, run.msa_mask, run.pair_mask, run.params,
                            run.msa_out, run.pair_out, sm, sp)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for i, (run, (m, z)) in enumerate(zip(runs, refs)):
        assert torch.equal(run.msa_out, m), i
        assert torch.equal(run.pair_out, z), i


def test_static_scratch_rejects_large_dims():
    dims, _, _ = dims_for("af2_initial")
    assert pe.workspace_bytes(dims, 1) > pe.static_scratch_bytes()
    small, inp = _inputs(54)
    run = BlockRun(small, inp)
    with pytest.raises(pe.PEError, match="static array holds"):
        pe.block_fwd_static(run.h, dims, run.msa, run.pair, run.msa_mask, run.pair_mask, run.params,
                            run.msa_out, run.pair_out, run.sm, run.sp)
