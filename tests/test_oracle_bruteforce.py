"""Pin every sub-op of the vectorised oracle to scalar-loop definitions."""
import numpy as np
import pytest

from oracle import evoformer as ev
from tests import brute
from tests.helpers import tiny_case, P_of

TOL = 1e-12


def _mixed_masks(inp, s, r):
    msa_mask = np.ones((s, r))
    msa_mask[1, 2] = 0.0
    msa_mask[:, r - 1] = 0.0          # a fully masked column (column attention sees no key)
    pair_mask = np.ones((r, r))
    pair_mask[0, 1] = 0.0
    pair_mask[:, r - 1] = 0.0
    pair_mask[r - 1, :] = 0.0
    return msa_mask, pair_mask


@pytest.fixture(scope="module")
def case():
    dims, table, n, inp = tiny_case(seed=3)
    mm, pm = _mixed_masks(inp, dims["s"], dims["r"])
    return dims, P_of(inp, table), inp, mm, pm


def test_row_attn(case):
    dims, P, inp, mm, pm = case
    u, _ = ev.row_attn_fwd(P, inp["msa"], inp["pair"], mm, dims)
    ref = brute.row_attn(P, inp["msa"], inp["pair"], mm, dims["h_msa"], dims["d_msa"], dims["ln_eps"])
    assert np.max(np.abs(u - ref)) < TOL


def test_col_attn(case):
    dims, P, inp, mm, pm = case
    u, _ = ev.col_attn_fwd(P, inp["msa"], mm, dims)
    ref = brute.col_attn(P, inp["msa"], mm, dims["h_msa"], dims["d_msa"], dims["ln_eps"])
    assert np.max(np.abs(u - ref)) < TOL


def test_col_global_attn():
    dims, table, n, inp = tiny_case(seed=4, col_global=1)
    P = P_of(inp, table)
    mm, _ = _mixed_masks(inp, dims["s"], dims["r"])
    u, _ = ev.col_global_attn_fwd(P, inp["msa"], mm, dims)
    ref = brute.col_global_attn(P, inp["msa"], mm, dims["h_msa"], dims["d_msa"], dims["ln_eps"])
    assert np.max(np.abs(u - ref)) < TOL


def test_transition(case):
    dims, P, inp, mm, pm = case
    u, _ = ev.transition_fwd(P, "mtrans", inp["msa"], dims)
    assert np.max(np.abs(u - brute.transition(P, "mtrans", inp["msa"], dims["ln_eps"]))) < TOL
    u, _ = ev.transition_fwd(P, "ptrans", inp["pair"], dims)
    assert np.max(np.abs(u - brute.transition(P, "ptrans", inp["pair"], dims["ln_eps"]))) < TOL


@pytest.mark.parametrize("outgoing", [True, False])
def test_tri_mul(case, outgoing):
    dims, P, inp, mm, pm = case
    pre = "tmo" if outgoing else "tmi"
    u, _ = ev.tri_mul_fwd(P, pre, inp["pair"], pm, dims, outgoing)
    ref = brute.tri_mul(P, pre, inp["pair"], pm, dims["ln_eps"], outgoing)
    assert np.max(np.abs(u - ref)) < TOL


@pytest.mark.parametrize("ending", [False, True])
def test_tri_attn(case, ending):
    dims, P, inp, mm, pm = case
    pre = "tae" if ending else "tas"
    f = ev.tri_attn_end_fwd if ending else ev.tri_attn_start_fwd
    u, _ = f(P, pre, inp["pair"], pm, dims)
    ref = brute.tri_attn(P, pre, inp["pair"], pm, dims["h_pair"], dims["d_pair"], dims["ln_eps"], ending)
    assert np.max(np.abs(u - ref)) < TOL


def test_opm(case):
    dims, P, inp, mm, pm = case
    u, _ = ev.opm_fwd(P, inp["msa"], mm, dims)
    ref = brute.opm(P, inp["msa"], mm, dims["c_opm"], dims["ln_eps"], dims["opm_eps"])
    assert np.max(np.abs(u - ref)) < TOL


@pytest.mark.parametrize("variant", [0, 1, 2])
@pytest.mark.parametrize("col_global", [0, 1])
def test_whole_block(col_global, variant):
    """All three orderings of Figure 1 against the scalar-loop composition."""
    dims, table, n, inp = tiny_case(seed=5, col_global=col_global, variant=variant)
    P = P_of(inp, table)
    mm, pm = _mixed_masks(inp, dims["s"], dims["r"])
    m, z, _, _ = ev.block_fwd(dims, inp["params"], inp["msa"], inp["pair"], mm, pm)
    mr, zr = brute.block(dims, P, inp["msa"], inp["pair"], mm, pm, variant=variant)
    assert np.max(np.abs(m - mr)) < 1e-11
    assert np.max(np.abs(z - zr)) < 1e-11


def test_stack_forward_chaining():
    """Which representation feeds which block in the trunk (Figure 2 caption: the extra MSA stack is made of
    Evoformer blocks and precedes the main ones): written out as two plain loops over the scalar-loop block.
    The extra blocks read (extra MSA, pair), the main blocks read (MSA, pair), the pair representation runs
    through all of them in order, each block has its own parameters, and the extra-MSA representation is
    dropped after the extra blocks.  The extra blocks use another channel width and row count than the main
    ones, so a block fed the wrong representation or the wrong parameter slice cannot even be evaluated."""
    from oracle.params import param_table, unpack
    from pe_inputs import make_inputs
    n_extra, n_main = 2, 2
    dims_m, table_m, n_m, inp = tiny_case(seed=31)
    dims_e = dict(dims_m, col_global=1, s=5, c_m=4)
    table_e, n_e = param_table(dims_e)
    inp_e = make_inputs(dims_e, table_e, n_e, ("none", 0), 32, n_blocks=n_extra)
    inp_m = make_inputs(dims_m, table_m, n_m, ("last_residues", 1), 33, n_blocks=n_main)
    extra_mask = inp_e["msa_mask"].copy()
    extra_mask[1, :] = 0.0
    params = np.concatenate([inp_e["params"], inp_m["params"]])
    res = ev.stack_fwd_bwd(n_extra, dims_e, n_main, dims_m, params, extra_msa=inp_e["msa"], msa=inp_m["msa"],
                           pair=inp_m["pair"], extra_mask=extra_mask, msa_mask=inp_m["msa_mask"],
                           pair_mask=inp_m["pair_mask"], d_msa_out=inp_m["d_msa_out"], d_pair_out=inp_m["d_pair_out"])
    e, m, z = inp_e["msa"], inp_m["msa"], inp_m["pair"]
    for b in range(n_extra):
        P = unpack(params[b * n_e:(b + 1) * n_e], table_e)
        e, z = brute.block(dims_e, P, e, z, extra_mask, inp_m["pair_mask"])
    for b in range(n_main):
        off = n_extra * n_e + b * n_m
        P = unpack(params[off:off + n_m], table_m)
        m, z = brute.block(dims_m, P, m, z, inp_m["msa_mask"], inp_m["pair_mask"])
    assert np.max(np.abs(res[0] - m)) < 1e-11
    assert np.max(np.abs(res[1] - z)) < 1e-11
    # planted mistakes are caught: main blocks in the other order, or the pair representation not passed on
    m2, z2 = inp_m["msa"], inp_m["pair"]
    for b in reversed(range(n_main)):
        off = n_extra * n_e + b * n_m
        m2, z2 = brute.block(dims_m, unpack(params[off:off + n_m], table_m), m2, z2, inp_m["msa_mask"], inp_m["pair_mask"])
    assert np.max(np.abs(res[0] - m2)) > 1e-3 and np.max(np.abs(res[1] - z2)) > 1e-3
