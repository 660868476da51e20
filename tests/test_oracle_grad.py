"""Central finite differences pin every hand-derived gradient of the oracle."""
import numpy as np
import pytest

from oracle import evoformer as ev
from oracle.params import param_table
from tests.helpers import tiny_case


def _loss(dims, params, msa, pair, mm, pm, wm, wz):
    m, z, _, _ = ev.block_fwd(dims, params, msa, pair, mm, pm, want_cache=False)
    return float((wm * m).sum() + (wz * z).sum())


def _fd(f, x, idx, h=1e-6):
    out = np.zeros(len(idx))
    flat = x.reshape(-1)
    for n, i in enumerate(idx):
        old = flat[i]
        flat[i] = old + h
        fp = f()
        flat[i] = old - h
        fm = f()
        flat[i] = old
        out[n] = (fp - fm) / (2 * h)
    return out


@pytest.mark.parametrize("variant", [0, 1, 2])
@pytest.mark.parametrize("col_global", [0, 1])
def test_block_gradients_fd(col_global, variant):
    dims, table, n, inp = tiny_case(seed=7, col_global=col_global, mask=("last_residues", 1), variant=variant)
    msa, pair, params = inp["msa"].copy(), inp["pair"].copy(), inp["params"].copy()
    mm, pm = inp["msa_mask"].copy(), inp["pair_mask"].copy()
    mm[1, 0] = 0.0
    pm[0, 2] = 0.0
    wm, wz = inp["d_msa_out"], inp["d_pair_out"]
    _, _, cache, _ = ev.block_fwd(dims, params, msa, pair, mm, pm)
    dm, dz, g, _ = ev.block_bwd(dims, cache, wm, wz)
    f = lambda: _loss(dims, params, msa, pair, mm, pm, wm, wz)
    rng = np.random.default_rng(0)
    # every parameter entry: a few elements each (all of the small ones)
    worst = 0.0
    for e in table:
        k = int(np.prod(e["shape"]))
        idx = e["offset"] + (np.arange(k) if k <= 6 else rng.choice(k, size=6, replace=False))
        num = _fd(f, params, idx)
        # row.ln_z.b has an exactly zero gradient (a per-head constant added to every
        # logit cancels in the softmax), so the scale also carries a global term
        scale = max(np.max(np.abs(g[e["offset"]:e["offset"] + k])), 1e-3 * np.max(np.abs(g)))
        err = np.max(np.abs(num - g[idx])) / scale
        worst = max(worst, err)
        assert err < 1e-6, (e["name"], err)
    idx = rng.choice(msa.size, size=40, replace=False)
    assert np.max(np.abs(_fd(f, msa, idx) - dm.reshape(-1)[idx])) / np.max(np.abs(dm)) < 1e-6
    idx = rng.choice(pair.size, size=60, replace=False)
    assert np.max(np.abs(_fd(f, pair, idx) - dz.reshape(-1)[idx])) / np.max(np.abs(dz)) < 1e-6


def _subop_fd(fwd, bwd, x, P, names, seed=0, extra_x=None):
    """fwd(P, x) -> (y, cache); bwd(P, G, dy, cache) -> dx (or tuple).  Checks dx and dP[names]."""
    rng = np.random.default_rng(seed)
    y, cache = fwd(P, x)
    w = rng.standard_normal(y.shape)
    G = {}
    dx = bwd(P, G, w, cache)
    f = lambda: float((w * fwd(P, x)[0]).sum())
    idx = rng.choice(x.size, size=min(30, x.size), replace=False)
    dx0 = dx[0] if isinstance(dx, tuple) else dx
    assert np.max(np.abs(_fd(f, x, idx) - dx0.reshape(-1)[idx])) / max(np.max(np.abs(dx0)), 1e-9) < 1e-6
    if extra_x is not None:
        idx = rng.choice(extra_x.size, size=min(30, extra_x.size), replace=False)
        assert np.max(np.abs(_fd(f, extra_x, idx) - dx[1].reshape(-1)[idx])) / np.max(np.abs(dx[1])) < 1e-6
    for nm in names:
        arr = P[nm]
        idx = rng.choice(arr.size, size=min(8, arr.size), replace=False)
        num = _fd(f, arr, idx)
        ana = np.asarray(G[nm]).reshape(-1)[idx]
        assert np.max(np.abs(num - ana)) / max(np.max(np.abs(G[nm])), 1e-3) < 1e-6, nm


def _P(dims, inp, table):
    # independent writable arrays per entry (views would alias the flat vector: fine, but copy for clarity)
    from oracle.params import unpack
    flat = inp["params"].copy()
    return unpack(flat, table)


def test_subops_fd():
    dims, table, n, inp = tiny_case(seed=11)
    P = _P(dims, inp, table)
    mm, pm = inp["msa_mask"].copy(), inp["pair_mask"].copy()
    mm[0, 1] = 0.0
    pm[1, 0] = 0.0
    msa, pair = inp["msa"].copy(), inp["pair"].copy()
    names = lambda pre: [e["name"] for e in table if e["name"].startswith(pre + ".")]
    _subop_fd(lambda P_, x: ev.row_attn_fwd(P_, x, pair, mm, dims),
              lambda P_, G, dy, c: ev.row_attn_bwd(P_, G, dy, c, dims), msa, P, names("row"), extra_x=pair)
    _subop_fd(lambda P_, x: ev.col_attn_fwd(P_, x, mm, dims),
              lambda P_, G, dy, c: ev.col_attn_bwd(P_, G, dy, c, dims), msa, P, names("col"))
    _subop_fd(lambda P_, x: ev.transition_fwd(P_, "mtrans", x, dims),
              lambda P_, G, dy, c: ev.transition_bwd(P_, G, "mtrans", dy, c), msa, P, names("mtrans"))
    _subop_fd(lambda P_, x: ev.opm_fwd(P_, x, mm, dims),
              lambda P_, G, dy, c: ev.opm_bwd(P_, G, dy, c, dims), msa, P, names("opm"))
    for pre, out in (("tmo", True), ("tmi", False)):
        _subop_fd(lambda P_, x: ev.tri_mul_fwd(P_, pre, x, pm, dims, out),
                  lambda P_, G, dy, c: ev.tri_mul_bwd(P_, G, pre, dy, c, out), pair, P, names(pre))
    _subop_fd(lambda P_, x: ev.tri_attn_start_fwd(P_, "tas", x, pm, dims),
              lambda P_, G, dy, c: ev.tri_attn_start_bwd(P_, G, "tas", dy, c, dims), pair, P, names("tas"))
    _subop_fd(lambda P_, x: ev.tri_attn_end_fwd(P_, "tae", x, pm, dims),
              lambda P_, G, dy, c: ev.tri_attn_end_bwd(P_, G, "tae", dy, c, dims), pair, P, names("tae"))
    _subop_fd(lambda P_, x: ev.transition_fwd(P_, "ptrans", x, dims),
              lambda P_, G, dy, c: ev.transition_bwd(P_, G, "ptrans", dy, c), pair, P, names("ptrans"))


def test_global_col_fd():
    dims, table, n, inp = tiny_case(seed=12, col_global=1)
    P = _P(dims, inp, table)
    mm = inp["msa_mask"].copy()
    mm[0, 1] = 0.0
    names = [e["name"] for e in table if e["name"].startswith("col.")]
    _subop_fd(lambda P_, x: ev.col_global_attn_fwd(P_, x, mm, dims),
              lambda P_, G, dy, c: ev.col_global_attn_bwd(P_, G, dy, c, dims), inp["msa"].copy(), P, names)


def test_stack_gradients_fd():
    """Two-block stack (1 extra + 1 main): gradient through the chained pair representation."""
    dims_m, table_m, n_m, inp = tiny_case(seed=13)
    dims_e = dict(dims_m, col_global=1, s=4)
    table_e, n_e = param_table(dims_e)
    from pe_inputs import make_inputs
    inp_e = make_inputs(dims_e, table_e, n_e, ("none", 0), 21)
    params = np.concatenate([inp_e["params"], inp["params"]])
    args = dict(extra_msa=inp_e["msa"], msa=inp["msa"], pair=inp["pair"], extra_mask=inp_e["msa_mask"],
                msa_mask=inp["msa_mask"], pair_mask=inp["pair_mask"],
                d_msa_out=inp["d_msa_out"], d_pair_out=inp["d_pair_out"])
    res = ev.stack_fwd_bwd(1, dims_e, 1, dims_m, params, **args)
    res2 = ev.stack_fwd_bwd(1, dims_e, 1, dims_m, params, recompute=False, **args)
    for a, b in zip(res, res2):
        assert np.array_equal(a, b)          # recompute == store-everything, bit for bit
    mo, zo, de, dm, dz, g = res

    def f():
        r_ = ev.stack_fwd_bwd(1, dims_e, 1, dims_m, params, **args)
        return float((args["d_msa_out"] * r_[0]).sum() + (args["d_pair_out"] * r_[1]).sum())
    rng = np.random.default_rng(1)
    idx = rng.choice(params.size, size=40, replace=False)
    num = _fd(f, params, idx)
    assert np.max(np.abs(num - g[idx]) / (np.abs(g[idx]) + 1e-3 * np.max(np.abs(g)))) < 1e-5
    em = args["extra_msa"]
    idx = rng.choice(em.size, size=20, replace=False)
    assert np.max(np.abs(_fd(f, em, idx) - de.reshape(-1)[idx])) / np.max(np.abs(de)) < 1e-6
    pz = args["pair"]
    idx = rng.choice(pz.size, size=20, replace=False)
    assert np.max(np.abs(_fd(f, pz, idx) - dz.reshape(-1)[idx])) / np.max(np.abs(dz)) < 1e-6


def test_relu_override_is_consistent():
    """With the on/off decision supplied explicitly the block is smooth in its inputs: the
    backward must be the exact derivative of that function (finite differences with the same
    fixed decisions), and supplying the default decisions changes nothing."""
    dims, table, n, inp = tiny_case(seed=17)
    msa, pair, params = inp["msa"].copy(), inp["pair"].copy(), inp["params"].copy()
    mm, pm, wm, wz = inp["msa_mask"], inp["pair_mask"], inp["d_msa_out"], inp["d_pair_out"]
    m0, z0, cache0, it0 = ev.block_fwd(dims, params, msa, pair, mm, pm)
    on = {"mtrans": it0["mtrans_pre"] > 0, "ptrans": it0["ptrans_pre"] > 0}
    m1, z1, cache1, _ = ev.block_fwd(dims, params, msa, pair, mm, pm, relu_on=on)
    assert np.array_equal(m0, m1) and np.array_equal(z0, z1)
    assert np.array_equal(ev.block_bwd(dims, cache0, wm, wz)[2], ev.block_bwd(dims, cache1, wm, wz)[2])
    # flip the decisions of the pre-activations closest to zero
    rng = np.random.default_rng(0)
    for k in ("mtrans", "ptrans"):
        a = it0[k + "_pre"]
        thr = np.quantile(np.abs(a), 0.1)
        on[k] = np.where(np.abs(a) < thr, rng.random(a.shape) < 0.5, a > 0)
    _, _, cache, _ = ev.block_fwd(dims, params, msa, pair, mm, pm, relu_on=on)
    dm, dz, g, _ = ev.block_bwd(dims, cache, wm, wz)

    def f():
        m, z, _, _ = ev.block_fwd(dims, params, msa, pair, mm, pm, want_cache=False, relu_on=on)
        return float((wm * m).sum() + (wz * z).sum())
    idx = rng.choice(params.size, size=60, replace=False)
    num = _fd(f, params, idx)
    assert np.max(np.abs(num - g[idx]) / (np.abs(g[idx]) + 1e-3 * np.max(np.abs(g)))) < 1e-5
    idx = rng.choice(msa.size, size=30, replace=False)
    assert np.max(np.abs(_fd(f, msa, idx) - dm.reshape(-1)[idx])) / np.max(np.abs(dm)) < 1e-6
    idx = rng.choice(pair.size, size=30, replace=False)
    assert np.max(np.abs(_fd(f, pair, idx) - dz.reshape(-1)[idx])) / np.max(np.abs(dz)) < 1e-6
