"""Closed forms, special cases and symmetry invariants that pin the oracle."""
import numpy as np
import pytest

from oracle import evoformer as ev
from oracle.params import param_table, unpack
from tests.helpers import tiny_case, P_of


def test_layernorm_moments():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 7, 16)) * 3 + 1
    eps = 1e-5
    y, _ = ev.ln_fwd(x, np.ones(16), np.zeros(16), eps)
    v = x.var(axis=-1)
    assert np.max(np.abs(y.mean(axis=-1))) < 1e-14
    assert np.max(np.abs(y.var(axis=-1) - v / (v + eps))) < 1e-13


def test_masked_softmax_properties():
    rng = np.random.default_rng(1)
    l = rng.standard_normal((3, 4, 6)) * 5
    kap = np.array([[1, 1, 0, 1, 0, 1], [0, 0, 0, 0, 0, 0], [1, 1, 1, 1, 1, 1]], dtype=float)[:, None, :]
    p = ev.masked_softmax(l, kap)
    assert np.allclose(p[0].sum(-1), 1.0, atol=1e-14) and np.allclose(p[2].sum(-1), 1.0, atol=1e-14)
    assert np.all(p[0][:, [2, 4]] == 0.0)
    assert np.all(p[1] == 0.0)                      # no valid key: zero output
    # unmasked case equals the textbook softmax
    e = np.exp(l[2] - l[2].max(-1, keepdims=True))
    assert np.allclose(p[2], e / e.sum(-1, keepdims=True), atol=1e-15)
    # shift invariance
    assert np.allclose(ev.masked_softmax(l + 100.0, kap), p, atol=1e-13)


def test_attention_reduces_to_textbook():
    """H=1, gate saturated, no bias, identity output projection: softmax(QK^T/sqrt d)V."""
    rng = np.random.default_rng(2)
    B, L, d = 2, 5, 4
    q, k, v = (rng.standard_normal((B, L, 1, d)) for _ in range(3))
    g = np.full((B, L, 1, d), 50.0)
    out, _ = ev.gated_attn_fwd(q, k, v, g, None, np.ones((B, L)))
    for b in range(B):
        S = q[b, :, 0] @ k[b, :, 0].T / np.sqrt(d)
        Pm = np.exp(S - S.max(-1, keepdims=True))
        Pm /= Pm.sum(-1, keepdims=True)
        assert np.allclose(out[b, :, 0], Pm @ v[b, :, 0], atol=1e-13)


def test_tri_mul_saturated_is_matmul():
    """Gates saturated, mask all ones: the contraction is a per-channel matrix product."""
    dims, table, n, inp = tiny_case(seed=2, mask=("none", 0))
    P = {k: v.copy() for k, v in P_of(inp, table).items()}
    for pre in ("tmo", "tmi"):
        for nm in ("ag", "bg"):
            P[pre + ".w_" + nm][:] = 0.0
            P[pre + ".b_" + nm][:] = 60.0
    z, pm = inp["pair"], inp["pair_mask"]
    for pre, out in (("tmo", True), ("tmi", False)):
        _, c = ev.tri_mul_fwd(P, pre, z, pm, dims, out)
        zh = c[1]
        A = zh @ P[pre + ".w_ap"] + P[pre + ".b_ap"]
        Bm = zh @ P[pre + ".w_bp"] + P[pre + ".b_bp"]
        x = np.stack([(A[:, :, ch] @ Bm[:, :, ch].T) if out else (A[:, :, ch].T @ Bm[:, :, ch])
                      for ch in range(A.shape[-1])], axis=-1)
        xh_ref, _ = ev.ln_fwd(x, P[pre + ".ln_out.g"], P[pre + ".ln_out.b"], dims["ln_eps"])
        assert np.allclose(c[11], xh_ref, atol=1e-11)


def test_tri_mul_incoming_is_outgoing_on_transposed_operands():
    rng = np.random.default_rng(3)
    r, c = 5, 3
    a, b = rng.standard_normal((r, r, c)), rng.standard_normal((r, r, c))
    x_in = np.einsum("kic,kjc->ijc", a, b)
    x_out_t = np.einsum("ikc,jkc->ijc", np.swapaxes(a, 0, 1), np.swapaxes(b, 0, 1))
    assert np.allclose(x_in, x_out_t, atol=1e-14)


def test_tri_attn_end_is_start_on_transpose():
    dims, table, n, inp = tiny_case(seed=4)
    P = P_of(inp, table)
    pm = inp["pair_mask"].copy()
    pm[0, 2] = 0.0
    z = inp["pair"]
    ue, _ = ev.tri_attn_end_fwd(P, "tae", z, pm, dims)
    P2 = dict(P)
    for k in list(P):
        if k.startswith("tae."):
            P2["tas." + k[4:]] = P[k]
    us, _ = ev.tri_attn_start_fwd(P2, "tas", np.swapaxes(z, 0, 1).copy(), pm.T.copy(), dims)
    assert np.allclose(ue, np.swapaxes(us, 0, 1), atol=1e-14)


def test_opm_properties():
    dims, table, n, inp = tiny_case(seed=5, mask=("none", 0))
    P = P_of(inp, table)
    m, mm = inp["msa"], inp["msa_mask"]
    u, c = ev.opm_fwd(P, m, mm, dims)
    perm = np.array([2, 0, 1])
    u2, _ = ev.opm_fwd(P, m[perm], mm[perm], dims)
    assert np.allclose(u, u2, atol=1e-13)                    # invariant to MSA-row order
    # s = 1: plain outer product divided by (eps + 1)
    u1, c1 = ev.opm_fwd(P, m[:1], mm[:1], dims)
    a, b = c1[3][0], c1[4][0]
    O = np.einsum("ip,jq->ijpq", a, b).reshape(dims["r"], dims["r"], -1) / (dims["opm_eps"] + 1.0)
    assert np.allclose(c1[6], O, atol=1e-14)
    # bilinear in (a, b): doubling w_a,b_a doubles the pre-projection tensor
    P2 = dict(P)
    P2["opm.w_a"], P2["opm.b_a"] = 2 * P["opm.w_a"], 2 * P["opm.b_a"]
    _, c2 = ev.opm_fwd(P2, m, mm, dims)
    assert np.allclose(c2[6], 2 * c[6], atol=1e-13)


def _blk(dims, inp, **over):
    a = dict(params=inp["params"], msa=inp["msa"], pair=inp["pair"],
             msa_mask=inp["msa_mask"], pair_mask=inp["pair_mask"])
    a.update(over)
    return ev.block_fwd(dims, a["params"], a["msa"], a["pair"], a["msa_mask"], a["pair_mask"])


def test_zero_output_projections_give_identity():
    dims, table, n, inp = tiny_case(seed=6)
    p = inp["params"].copy()
    for e in table:
        if e["name"].split(".")[-1] in ("w_o", "b_o", "w2", "b2"):
            k = int(np.prod(e["shape"]))
            p[e["offset"]:e["offset"] + k] = 0.0
    m, z, _, _ = _blk(dims, inp, params=p)
    assert np.array_equal(m, inp["msa"]) and np.array_equal(z, inp["pair"])


def test_block_orderings_differ_only_through_the_outer_product_mean():
    """Figure 1: the three blocks are the same stacks with the outer product mean in different
    places.  With its output projection zeroed they coincide; with it active the AlphaFold2
    ordering is the Parallel block's pair stack applied to pair + opm(msa_out), and the Multimer
    ordering is the Parallel block applied to the pair input pair + opm(msa_in) with the final
    outer-product term left out."""
    dims, table, n, inp = tiny_case(seed=12)
    p0 = inp["params"].copy()
    for e in table:
        if e["name"] in ("opm.w_o", "opm.b_o"):
            k = int(np.prod(e["shape"]))
            p0[e["offset"]:e["offset"] + k] = 0.0
    outs = [_blk(dict(dims, variant=v), inp, params=p0)[:2] for v in (0, 1, 2)]
    for m, z in outs[1:]:
        assert np.array_equal(m, outs[0][0]) and np.array_equal(z, outs[0][1])
    m0, z0, _, i0 = _blk(dims, inp)
    # AlphaFold2 ordering from Parallel pieces
    _, _, _, ia = _blk(dims, inp, pair=inp["pair"] + i0["opm"])
    m1, z1, _, _ = _blk(dict(dims, variant=1), inp)
    assert np.array_equal(m1, m0) and np.allclose(z1, ia["z5"], atol=1e-12)
    assert not np.allclose(z1, z0, atol=1e-3)
    # Multimer ordering from Parallel pieces: opm(msa_in) from a block whose MSA stack is the identity
    pid = inp["params"].copy()
    for e in table:
        if e["name"] in ("row.w_o", "row.b_o", "col.w_o", "col.b_o", "mtrans.w2", "mtrans.b2"):
            k = int(np.prod(e["shape"]))
            pid[e["offset"]:e["offset"] + k] = 0.0
    _, _, _, iid = _blk(dims, inp, params=pid)
    assert np.array_equal(iid["m3"], inp["msa"])
    mb, _, _, ib = _blk(dims, inp, pair=inp["pair"] + iid["opm"])
    m2, z2, _, _ = _blk(dict(dims, variant=2), inp)
    assert np.allclose(m2, mb, atol=1e-12) and np.allclose(z2, ib["z5"], atol=1e-12)
    assert not np.allclose(m2, m0, atol=1e-3)


@pytest.mark.parametrize("col_global", [0, 1])
def test_residue_permutation_equivariance(col_global):
    dims, table, n, inp = tiny_case(seed=7, col_global=col_global, mask=("last_residues", 1))
    perm = np.array([2, 0, 3, 1])
    m, z, _, _ = _blk(dims, inp)
    m2, z2, _, _ = _blk(dims, inp, msa=inp["msa"][:, perm], pair=inp["pair"][perm][:, perm],
                        msa_mask=inp["msa_mask"][:, perm], pair_mask=inp["pair_mask"][perm][:, perm])
    assert np.allclose(m2, m[:, perm], atol=1e-12)
    assert np.allclose(z2, z[perm][:, perm], atol=1e-12)


@pytest.mark.parametrize("col_global", [0, 1])
def test_msa_row_permutation(col_global):
    dims, table, n, inp = tiny_case(seed=8, col_global=col_global)
    mm = inp["msa_mask"].copy()
    mm[1, 0] = 0.0
    perm = np.array([1, 2, 0])
    m, z, _, _ = _blk(dims, inp, msa_mask=mm)
    m2, z2, _, _ = _blk(dims, inp, msa=inp["msa"][perm], msa_mask=mm[perm])
    assert np.allclose(m2, m[perm], atol=1e-12)
    assert np.allclose(z2, z, atol=1e-12)


def test_padding_isolation():
    """Outputs at unmasked residues do not depend on inputs at masked residues."""
    dims, table, n, inp = tiny_case(seed=9, mask=("last_residues", 1))
    r = dims["r"]
    rng = np.random.default_rng(0)
    msa2, pair2 = inp["msa"].copy(), inp["pair"].copy()
    msa2[:, r - 1] = rng.standard_normal(msa2[:, r - 1].shape)
    pair2[r - 1, :] = rng.standard_normal(pair2[r - 1].shape)
    pair2[:, r - 1] = rng.standard_normal(pair2[:, r - 1].shape)
    m, z, _, _ = _blk(dims, inp)
    m2, z2, _, _ = _blk(dims, inp, msa=msa2, pair=pair2)
    assert np.allclose(m2[:, :r - 1], m[:, :r - 1], atol=1e-12)
    assert np.allclose(z2[:r - 1, :r - 1], z[:r - 1, :r - 1], atol=1e-12)


def test_branch_independence():
    """Section "Parallel Evoformer": the branches evolve independently inside a block."""
    dims, table, n, inp = tiny_case(seed=10)
    rng = np.random.default_rng(0)
    m, z, _, it = _blk(dims, inp)
    # perturb every pair-branch parameter: msa_out and the OPM term unchanged
    p2 = inp["params"].copy()
    for e in table:
        if e["name"].split(".")[0] in ("tmo", "tmi", "tas", "tae", "ptrans"):
            k = int(np.prod(e["shape"]))
            p2[e["offset"]:e["offset"] + k] += rng.standard_normal(k)
    m2, z2, _, it2 = _blk(dims, inp, params=p2)
    assert np.array_equal(m2, m) and np.array_equal(it2["opm"], it["opm"])
    assert not np.allclose(it2["z5"], it["z5"])
    # perturb the MSA input: the pair branch's part z5 is unchanged, pair_out - z5 is the OPM term
    m3, z3, _, it3 = _blk(dims, inp, msa=inp["msa"] + 1.0)
    assert np.array_equal(it3["z5"], it["z5"])
    assert np.allclose(z3 - it3["z5"], it3["opm"], atol=1e-12)
    # the row-attention bias reads the INPUT pair representation: changing pair-branch
    # parameters (hence every updated pair tensor) left msa_out unchanged above.


def test_dpair_in_decomposition():
    """Section "Branch Parallelism": the gradient of the input pair representation is the sum
    of the pair-branch term and the row-attention-bias term."""
    dims, table, n, inp = tiny_case(seed=11)
    _, _, cache, _ = _blk(dims, inp)
    wm, wz = inp["d_msa_out"], inp["d_pair_out"]
    dm, dz, g, parts = ev.block_bwd(dims, cache, wm, wz)
    assert np.allclose(dz, parts["dz_pair_branch"] + parts["dz_bias"], atol=0)
    # zero upstream pair cotangent: pair-branch term vanishes, OPM term too -> only bias term from d_msa_out
    dm0, dz0, g0, parts0 = ev.block_bwd(dims, cache, wm, np.zeros_like(wz))
    assert np.all(parts0["dz_pair_branch"] == 0.0)
    assert np.max(np.abs(dz0)) > 0
    # zero upstream MSA cotangent: bias term comes only through the OPM path
    dm1, dz1, g1, parts1 = ev.block_bwd(dims, cache, np.zeros_like(wm), wz)
    assert np.allclose(parts1["dz_pair_branch"], parts["dz_pair_branch"], atol=1e-13)
    assert np.allclose(parts0["dz_bias"] + parts1["dz_bias"], parts["dz_bias"], atol=1e-12)


def _paper_settings():
    import os
    out = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "paper_settings.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def test_workload_shapes_are_the_papers():
    """The benchmark and test workloads carry the shapes the paper prints (Table 1, caption of Table 5)."""
    from pe_inputs import dims_for
    g = _paper_settings()
    ini, ext, fin, exf = (dims_for(k)[0] for k in ("af2_initial", "extra_msa", "af2_finetune", "extra_msa_finetune"))
    assert (ini["r"], ini["s"], ext["s"]) == (g["initial_training.N_res"], g["initial_training.N_seq"],
                                             g["initial_training.N_extra_seq"])
    assert (fin["r"], fin["s"], exf["s"], exf["r"]) == (g["fine_tuning.N_res"], g["fine_tuning.N_seq"],
                                                       g["fine_tuning.N_extra_seq"], g["fine_tuning.N_res"])
    assert (ini["h_msa"], ini["s"], ini["r"], ini["c_m"], ini["c_z"]) == (g["table5.head"], g["table5.N_seq"],
                                                                         g["table5.N_res"], g["table5.C_m"], g["table5.C_z"])
    assert ext["r"] == ini["r"] and ext["c_z"] == ini["c_z"]


def test_param_count_matches_published_structure():
    """The trunk (48 main + 4 extra-MSA blocks, Section "Parallel Evoformer") holds most of the
    93 M parameters the paper quotes for the whole model (Introduction)."""
    from pe_inputs import dims_for
    g = _paper_settings()
    n_main = param_table(dims_for("af2_initial")[0])[1]
    n_extra = param_table(dims_for("extra_msa")[0])[1]
    total = int(g["trunk.main_blocks"]) * n_main + int(g["trunk.extra_blocks"]) * n_extra
    assert total == 90_642_944
    assert 0.9 * g["model.parameters"] < total < g["model.parameters"]
