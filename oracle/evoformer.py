"""Float64 CPU oracle of the Parallel Evoformer block (TEST INFRASTRUCTURE).

Plain numpy, float64, no blocking or fusion.  The composition of the block is
the paper's: Section "Parallel Evoformer" and Figure 1(c) (MSA branch and pair
branch evolve independently, outer product mean at the end of the block) and
Section "Branch Parallelism" (which tensors cross between the branches in the
forward and backward pass).  The paper names the sub-operations (Section
"Evoformer") and defers their definitions to AlphaFold2; the formulas used
here are the ones stated in this repository's design notes, each written out
as its plain definition.  The backward pass is derived by hand.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this file.  It shares no code with the HIP path.

Every function below is pinned by tests that do not retype its formula:
scalar-loop brute force, central finite differences, closed forms and
symmetry invariants (see tests/test_oracle_*.py).
"""
import numpy as np

from .params import param_table, unpack


# --------------------------------------------------------------------------
# primitives
# --------------------------------------------------------------------------
def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def ln_fwd(x, g, b, eps):
    """LayerNorm over the last axis, biased variance."""
    mu = x.mean(axis=-1, keepdims=True)
    xc = x - mu
    var = (xc * xc).mean(axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xh = xc * rstd
    return xh * g + b, (xh, rstd, g)


def ln_bwd(dy, cache):
    xh, rstd, g = cache
    lead = tuple(range(dy.ndim - 1))
    dg = (dy * xh).sum(axis=lead)
    db = dy.sum(axis=lead)
    dxh = dy * g
    dx = (dxh - dxh.mean(axis=-1, keepdims=True)
          - xh * (dxh * xh).mean(axis=-1, keepdims=True)) * rstd
    return dx, dg, db


def lin_fwd(x, w, b=None):
    y = x @ w
    return y if b is None else y + b


def lin_bwd(x, w, dy, has_bias=True):
    """Returns dx, dw, db for y = x w + b (sums over all leading axes)."""
    k, n = w.shape
    dx = dy @ w.T
    dw = x.reshape(-1, k).T @ dy.reshape(-1, n)
    db = dy.reshape(-1, n).sum(axis=0) if has_bias else None
    return dx, dw, db


def masked_softmax(l, kappa):
    """Softmax over the last axis restricted to keys with kappa == 1.
    Masked keys get weight exactly 0; a row with no valid key is all zero."""
    valid = kappa > 0
    lm = np.where(valid, l, -np.inf)
    mx = lm.max(axis=-1, keepdims=True)
    mx = np.where(np.isfinite(mx), mx, 0.0)
    e = np.where(valid, np.exp(np.where(valid, l, 0.0) - mx), 0.0)
    den = e.sum(axis=-1, keepdims=True)
    return np.where(den > 0, e / np.where(den > 0, den, 1.0), 0.0)


def softmax_bwd(p, dp):
    return p * (dp - (p * dp).sum(axis=-1, keepdims=True))


# --------------------------------------------------------------------------
# gated attention core
#   q,k,v,g: [B, L, H, d]; bias: [H, L, L] or None (shared over B);
#   kappa: [B, L] key mask
# --------------------------------------------------------------------------
def gated_attn_fwd(q, k, v, g, bias, kappa):
    B, L, H, d = q.shape
    o = np.zeros_like(q)
    ps = []
    for h in range(H):
        l = q[:, :, h] @ np.swapaxes(k[:, :, h], 1, 2) / np.sqrt(d)        # [B, Lq, Lk]
        if bias is not None:
            l = l + bias[h][None]
        p = masked_softmax(l, kappa[:, None, :])
        o[:, :, h] = p @ v[:, :, h]
        ps.append(p)
    sg = sigmoid(g)
    return sg * o, (q, k, v, sg, o, ps, bias is not None)


def gated_attn_bwd(dout, cache):
    q, k, v, sg, o, ps, has_bias = cache
    B, L, H, d = q.shape
    do = dout * sg
    dg = dout * o * sg * (1.0 - sg)
    dq, dk, dv = np.zeros_like(q), np.zeros_like(k), np.zeros_like(v)
    dbias = np.zeros((H, L, L)) if has_bias else None
    for h in range(H):
        p = ps[h]
        dv[:, :, h] = np.swapaxes(p, 1, 2) @ do[:, :, h]
        dp = do[:, :, h] @ np.swapaxes(v[:, :, h], 1, 2)
        dl = softmax_bwd(p, dp)
        dq[:, :, h] = dl @ k[:, :, h] / np.sqrt(d)
        dk[:, :, h] = np.swapaxes(dl, 1, 2) @ q[:, :, h] / np.sqrt(d)
        if has_bias:
            dbias[h] = dl.sum(axis=0)
    return dq, dk, dv, dg, dbias


# --------------------------------------------------------------------------
# attention sub-ops.  x: [B, L, c]; returns the update (residual added by caller)
# --------------------------------------------------------------------------
def _attn_update_fwd(P, pre, xh, H, d, bias, kappa):
    B, L, _ = xh.shape
    q = lin_fwd(xh, P[pre + ".w_q"]).reshape(B, L, H, d)
    k = lin_fwd(xh, P[pre + ".w_k"]).reshape(B, L, H, d)
    v = lin_fwd(xh, P[pre + ".w_v"]).reshape(B, L, H, d)
    g = lin_fwd(xh, P[pre + ".w_g"], P[pre + ".b_g"]).reshape(B, L, H, d)
    og, core = gated_attn_fwd(q, k, v, g, bias, kappa)
    og2 = og.reshape(B, L, H * d)
    upd = lin_fwd(og2, P[pre + ".w_o"], P[pre + ".b_o"])
    return upd, (xh, og2, core)


def _attn_update_bwd(P, G, pre, dupd, cache, H, d):
    xh, og2, core = cache
    B, L, _ = xh.shape
    dog, G[pre + ".w_o"], G[pre + ".b_o"] = lin_bwd(og2, P[pre + ".w_o"], dupd)
    dq, dk, dv, dg, dbias = gated_attn_bwd(dog.reshape(B, L, H, d), core)
    dxh = 0.0
    for nm, dt in (("q", dq), ("k", dk), ("v", dv), ("g", dg)):
        dx_, G[pre + ".w_" + nm], db_ = lin_bwd(xh, P[pre + ".w_" + nm], dt.reshape(B, L, H * d),
                                                has_bias=(nm == "g"))
        if nm == "g":
            G[pre + ".b_g"] = db_
        dxh = dxh + dx_
    return dxh, dbias


def row_attn_fwd(P, m, pair_in, msa_mask, dims):
    """MSA row-wise gated self-attention with pair bias (update only)."""
    H, d, eps = dims["h_msa"], dims["d_msa"], dims["ln_eps"]
    mh, c_m = ln_fwd(m, P["row.ln_m.g"], P["row.ln_m.b"], eps)
    zh, c_z = ln_fwd(pair_in, P["row.ln_z.g"], P["row.ln_z.b"], eps)
    bias = np.transpose(lin_fwd(zh, P["row.w_bias"]), (2, 0, 1))      # [H, r, r]
    upd, c_a = _attn_update_fwd(P, "row", mh, H, d, bias, msa_mask)
    return upd, (c_m, c_z, zh, c_a)


def row_attn_bwd(P, G, dupd, cache, dims):
    H, d = dims["h_msa"], dims["d_msa"]
    c_m, c_z, zh, c_a = cache
    dmh, dbias = _attn_update_bwd(P, G, "row", dupd, c_a, H, d)
    dm, G["row.ln_m.g"], G["row.ln_m.b"] = ln_bwd(dmh, c_m)
    dbz = np.transpose(dbias, (1, 2, 0))                                # [r, r, H]
    dzh, G["row.w_bias"], _ = lin_bwd(zh, P["row.w_bias"], dbz, has_bias=False)
    dz, G["row.ln_z.g"], G["row.ln_z.b"] = ln_bwd(dzh, c_z)
    return dm, dz


def col_attn_fwd(P, m, msa_mask, dims):
    """MSA column-wise gated self-attention: attention along s for each residue."""
    H, d, eps = dims["h_msa"], dims["d_msa"], dims["ln_eps"]
    mh, c_m = ln_fwd(m, P["col.ln.g"], P["col.ln.b"], eps)
    mt = np.swapaxes(mh, 0, 1)                                          # [r, s, c]
    upd, c_a = _attn_update_fwd(P, "col", mt, H, d, None, msa_mask.T)
    return np.swapaxes(upd, 0, 1), (c_m, c_a)


def col_attn_bwd(P, G, dupd, cache, dims):
    H, d = dims["h_msa"], dims["d_msa"]
    c_m, c_a = cache
    dmt, _ = _attn_update_bwd(P, G, "col", np.swapaxes(dupd, 0, 1), c_a, H, d)
    dm, G["col.ln.g"], G["col.ln.b"] = ln_bwd(np.swapaxes(dmt, 0, 1), c_m)
    return dm


def col_global_attn_fwd(P, m, msa_mask, dims):
    """Global column attention of the extra-MSA blocks: one mask-averaged query
    per (residue, head), single-head keys and values."""
    H, d, eps = dims["h_msa"], dims["d_msa"], dims["ln_eps"]
    s, r, _ = m.shape
    mh, c_m = ln_fwd(m, P["col.ln.g"], P["col.ln.b"], eps)
    q = lin_fwd(mh, P["col.w_q"]).reshape(s, r, H, d)
    k = lin_fwd(mh, P["col.w_k"])                                        # [s, r, d]
    v = lin_fwd(mh, P["col.w_v"])
    g = lin_fwd(mh, P["col.w_g"], P["col.b_g"]).reshape(s, r, H, d)
    den = msa_mask.sum(axis=0) + 1e-10                                   # [r]
    qbar = np.einsum("si,sihd->ihd", msa_mask, q) / den[:, None, None]   # [r, H, d]
    l = np.einsum("ihd,tid->iht", qbar, k) / np.sqrt(d)                  # [r, H, s]
    p = masked_softmax(l, msa_mask.T[:, None, :])
    o = np.einsum("iht,tid->ihd", p, v)                                  # [r, H, d]
    sg = sigmoid(g)
    out = (sg * o[None]).reshape(s, r, H * d)
    upd = lin_fwd(out, P["col.w_o"], P["col.b_o"])
    return upd, (c_m, mh, q, k, v, sg, den, qbar, p, o, out, msa_mask)


def col_global_attn_bwd(P, G, dupd, cache, dims):
    H, d = dims["h_msa"], dims["d_msa"]
    c_m, mh, q, k, v, sg, den, qbar, p, o, out, msa_mask = cache
    s, r, _ = mh.shape
    dout, G["col.w_o"], G["col.b_o"] = lin_bwd(out, P["col.w_o"], dupd)
    dout = dout.reshape(s, r, H, d)
    do = (dout * sg).sum(axis=0)                                         # [r, H, d]
    dg = dout * o[None] * sg * (1.0 - sg)
    dv = np.einsum("iht,ihd->tid", p, do)
    dp = np.einsum("ihd,tid->iht", do, v)
    dl = softmax_bwd(p, dp)
    dqbar = np.einsum("iht,tid->ihd", dl, k) / np.sqrt(d)
    dk = np.einsum("iht,ihd->tid", dl, qbar) / np.sqrt(d)
    dq = msa_mask[:, :, None, None] * (dqbar / den[:, None, None])[None]
    dmh = 0.0
    for nm, dt in (("q", dq.reshape(s, r, H * d)), ("k", dk), ("v", dv), ("g", dg.reshape(s, r, H * d))):
        dx_, G["col.w_" + nm], db_ = lin_bwd(mh, P["col.w_" + nm], dt, has_bias=(nm == "g"))
        if nm == "g":
            G["col.b_g"] = db_
        dmh = dmh + dx_
    dm, G["col.ln.g"], G["col.ln.b"] = ln_bwd(dmh, c_m)
    return dm


def tri_attn_start_fwd(P, pre, z, pair_mask, dims):
    """Triangle self-attention around the starting node: for each row i,
    query (i,j) attends over keys (i,k) with bias from (j,k)."""
    H, d, eps = dims["h_pair"], dims["d_pair"], dims["ln_eps"]
    zh, c_z = ln_fwd(z, P[pre + ".ln.g"], P[pre + ".ln.b"], eps)
    bias = np.transpose(lin_fwd(zh, P[pre + ".w_bias"]), (2, 0, 1))
    upd, c_a = _attn_update_fwd(P, pre, zh, H, d, bias, pair_mask)
    return upd, (c_z, zh, c_a)


def tri_attn_start_bwd(P, G, pre, dupd, cache, dims):
    H, d = dims["h_pair"], dims["d_pair"]
    c_z, zh, c_a = cache
    dzh, dbias = _attn_update_bwd(P, G, pre, dupd, c_a, H, d)
    dzh2, G[pre + ".w_bias"], _ = lin_bwd(zh, P[pre + ".w_bias"], np.transpose(dbias, (1, 2, 0)),
                                          has_bias=False)
    dz, G[pre + ".ln.g"], G[pre + ".ln.b"] = ln_bwd(dzh + dzh2, c_z)
    return dz


def tri_attn_end_fwd(P, pre, z, pair_mask, dims):
    """Triangle self-attention around the ending node: the starting-node
    operation applied to the pair tensor with its two residue axes swapped."""
    upd, c = tri_attn_start_fwd(P, pre, np.swapaxes(z, 0, 1), pair_mask.T, dims)
    return np.swapaxes(upd, 0, 1), c


def tri_attn_end_bwd(P, G, pre, dupd, cache, dims):
    dz = tri_attn_start_bwd(P, G, pre, np.swapaxes(dupd, 0, 1), cache, dims)
    return np.swapaxes(dz, 0, 1)


# --------------------------------------------------------------------------
# transition
# --------------------------------------------------------------------------
def transition_fwd(P, pre, x, dims, relu_on=None):
    """LN -> Linear -> ReLU -> Linear.  `relu_on` (bool array, optional) overrides the
    ReLU on/off decision a > 0: h = a where relu_on else 0.  It exists for parity tests
    of reduced-precision implementations, where the sign of a pre-activation within the
    implementation's rounding error of zero is not uniquely determined; the default
    (None) is the plain definition."""
    xh, c_ln = ln_fwd(x, P[pre + ".ln.g"], P[pre + ".ln.b"], dims["ln_eps"])
    a = lin_fwd(xh, P[pre + ".w1"], P[pre + ".b1"])
    on = (a > 0) if relu_on is None else relu_on
    h = np.where(on, a, 0.0)
    return lin_fwd(h, P[pre + ".w2"], P[pre + ".b2"]), (c_ln, xh, a, h, on)


def transition_bwd(P, G, pre, dupd, cache):
    c_ln, xh, a, h, on = cache
    dh, G[pre + ".w2"], G[pre + ".b2"] = lin_bwd(h, P[pre + ".w2"], dupd)
    da = dh * on
    dxh, G[pre + ".w1"], G[pre + ".b1"] = lin_bwd(xh, P[pre + ".w1"], da)
    dx, G[pre + ".ln.g"], G[pre + ".ln.b"] = ln_bwd(dxh, c_ln)
    return dx


# --------------------------------------------------------------------------
# triangle multiplicative update
# --------------------------------------------------------------------------
def tri_contract(a, b, outgoing):
    """x_ijc = sum_k a_ikc b_jkc (outgoing) or sum_k a_kic b_kjc (incoming),
    written as one matrix product per channel."""
    at, bt = (np.ascontiguousarray(np.transpose(t, (2, 0, 1))) for t in (a, b))   # [c, ., .]
    xt = at @ np.swapaxes(bt, 1, 2) if outgoing else np.swapaxes(at, 1, 2) @ bt
    return np.transpose(xt, (1, 2, 0))


def tri_contract_bwd(dx, a, b, outgoing):
    at, bt, dxt = (np.ascontiguousarray(np.transpose(t, (2, 0, 1))) for t in (a, b, dx))
    if outgoing:        # x = a b^T per channel
        dat, dbt = dxt @ bt, np.swapaxes(dxt, 1, 2) @ at
    else:               # x = a^T b per channel
        dat, dbt = bt @ np.swapaxes(dxt, 1, 2), at @ dxt
    return np.transpose(dat, (1, 2, 0)), np.transpose(dbt, (1, 2, 0))


def tri_mul_fwd(P, pre, z, pair_mask, dims, outgoing):
    eps = dims["ln_eps"]
    zh, c_in = ln_fwd(z, P[pre + ".ln_in.g"], P[pre + ".ln_in.b"], eps)
    rho = pair_mask[:, :, None]
    ap = lin_fwd(zh, P[pre + ".w_ap"], P[pre + ".b_ap"])
    sa = sigmoid(lin_fwd(zh, P[pre + ".w_ag"], P[pre + ".b_ag"]))
    bp = lin_fwd(zh, P[pre + ".w_bp"], P[pre + ".b_bp"])
    sb = sigmoid(lin_fwd(zh, P[pre + ".w_bg"], P[pre + ".b_bg"]))
    a = rho * sa * ap
    b = rho * sb * bp
    g = sigmoid(lin_fwd(zh, P[pre + ".w_g"], P[pre + ".b_g"]))
    x = tri_contract(a, b, outgoing)
    xh, c_out = ln_fwd(x, P[pre + ".ln_out.g"], P[pre + ".ln_out.b"], eps)
    u = lin_fwd(xh, P[pre + ".w_o"], P[pre + ".b_o"])
    return g * u, (c_in, zh, rho, ap, sa, bp, sb, a, b, g, c_out, xh, u)


def tri_mul_bwd(P, G, pre, dupd, cache, outgoing):
    c_in, zh, rho, ap, sa, bp, sb, a, b, g, c_out, xh, u = cache
    du = dupd * g
    dgraw = dupd * u * g * (1.0 - g)
    dxh, G[pre + ".w_o"], G[pre + ".b_o"] = lin_bwd(xh, P[pre + ".w_o"], du)
    dx, G[pre + ".ln_out.g"], G[pre + ".ln_out.b"] = ln_bwd(dxh, c_out)
    da, db = tri_contract_bwd(dx, a, b, outgoing)
    dzh, G[pre + ".w_g"], G[pre + ".b_g"] = lin_bwd(zh, P[pre + ".w_g"], dgraw)
    for nm, dt in (("ap", da * rho * sa), ("ag", da * rho * ap * sa * (1.0 - sa)),
                   ("bp", db * rho * sb), ("bg", db * rho * bp * sb * (1.0 - sb))):
        dx_, G[pre + ".w_" + nm], G[pre + ".b_" + nm] = lin_bwd(zh, P[pre + ".w_" + nm], dt)
        dzh = dzh + dx_
    dz, G[pre + ".ln_in.g"], G[pre + ".ln_in.b"] = ln_bwd(dzh, c_in)
    return dz


# --------------------------------------------------------------------------
# outer product mean
# --------------------------------------------------------------------------
def outer_sum(a, b):
    """O_ijpq = sum_s a_sip b_sjq as one matrix product over s."""
    s, r, c = a.shape
    O = a.reshape(s, r * c).T @ b.reshape(s, r * c)                      # [(i,p), (j,q)]
    return np.transpose(O.reshape(r, c, r, c), (0, 2, 1, 3))


def outer_sum_bwd(dO, a, b):
    s, r, c = a.shape
    dOm = np.transpose(dO, (0, 2, 1, 3)).reshape(r * c, r * c)          # [(i,p), (j,q)]
    da = (b.reshape(s, r * c) @ dOm.T).reshape(s, r, c)
    db = (a.reshape(s, r * c) @ dOm).reshape(s, r, c)
    return da, db


def opm_fwd(P, m, msa_mask, dims):
    """O_ij = sum_s a_si (x) b_sj / (eps_o + sum_s mu_si mu_sj), then Linear."""
    s, r, _ = m.shape
    c_o = dims["c_opm"]
    mh, c_ln = ln_fwd(m, P["opm.ln.g"], P["opm.ln.b"], dims["ln_eps"])
    mu = msa_mask[:, :, None]
    a = mu * lin_fwd(mh, P["opm.w_a"], P["opm.b_a"])
    b = mu * lin_fwd(mh, P["opm.w_b"], P["opm.b_b"])
    norm = dims["opm_eps"] + msa_mask.T @ msa_mask                      # [r, r]
    O = outer_sum(a, b) / norm[:, :, None, None]
    Of = O.reshape(r, r, c_o * c_o)
    return lin_fwd(Of, P["opm.w_o"], P["opm.b_o"]), (c_ln, mh, mu, a, b, norm, Of)


def opm_bwd(P, G, dupd, cache, dims):
    c_ln, mh, mu, a, b, norm, Of = cache
    r = Of.shape[0]
    c_o = dims["c_opm"]
    dOf, G["opm.w_o"], G["opm.b_o"] = lin_bwd(Of, P["opm.w_o"], dupd)
    dO = dOf.reshape(r, r, c_o, c_o) / norm[:, :, None, None]
    da, db = outer_sum_bwd(dO, a, b)
    dmh_a, G["opm.w_a"], G["opm.b_a"] = lin_bwd(mh, P["opm.w_a"], da * mu)
    dmh_b, G["opm.w_b"], G["opm.b_b"] = lin_bwd(mh, P["opm.w_b"], db * mu)
    dm, G["opm.ln.g"], G["opm.ln.b"] = ln_bwd(dmh_a + dmh_b, c_ln)
    return dm


# --------------------------------------------------------------------------
# the block
# --------------------------------------------------------------------------
def _msa_stack_fwd(P, C, dims, msa, bias_pair, msa_mask, relu_on):
    u, C["row"] = row_attn_fwd(P, msa, bias_pair, msa_mask, dims)
    m1 = msa + u
    if dims["col_global"]:
        u, C["col"] = col_global_attn_fwd(P, m1, msa_mask, dims)
    else:
        u, C["col"] = col_attn_fwd(P, m1, msa_mask, dims)
    m2 = m1 + u
    u, C["mtrans"] = transition_fwd(P, "mtrans", m2, dims, relu_on.get("mtrans"))
    return m1, m2, m2 + u


def _pair_stack_fwd(P, C, dims, z0, pair_mask, relu_on):
    u, C["tmo"] = tri_mul_fwd(P, "tmo", z0, pair_mask, dims, True)
    z1 = z0 + u
    u, C["tmi"] = tri_mul_fwd(P, "tmi", z1, pair_mask, dims, False)
    z2 = z1 + u
    u, C["tas"] = tri_attn_start_fwd(P, "tas", z2, pair_mask, dims)
    z3 = z2 + u
    u, C["tae"] = tri_attn_end_fwd(P, "tae", z3, pair_mask, dims)
    z4 = z3 + u
    u, C["ptrans"] = transition_fwd(P, "ptrans", z4, dims, relu_on.get("ptrans"))
    return z1, z2, z3, z4, z4 + u


def block_fwd(dims, params, msa, pair, msa_mask, pair_mask, want_cache=True, relu_on=None):
    """Evoformer block forward, the three orderings of Figure 1 selected by
    dims["variant"] (default 0).  MSA stack: row attention biased by a pair
    representation, column attention, transition.  Pair stack: triangle
    multiplication outgoing then incoming, triangle attention starting then
    ending node, transition.  They differ in where the outer product mean sits:
      0  Parallel Evoformer, Figure 1(c), Section "Parallel Evoformer": both stacks
         read the block's inputs; the outer product mean of the MSA stack's OUTPUT
         is added to the pair stack's output at the end.
      1  AlphaFold2, Figure 1(a): the outer product mean of the MSA stack's output
         is added to the pair representation BEFORE the pair stack (serial).
      2  AlphaFold-Multimer, Figure 1(b): the outer product mean of the block's
         INPUT MSA representation is added to the pair representation at the start;
         the MSA stack (its row-attention bias) and the pair stack both read that sum.
    relu_on: optional {"mtrans": bool array, "ptrans": bool array}, see transition_fwd."""
    relu_on = relu_on or {}
    variant = dims.get("variant", 0)
    table, _ = param_table(dims)
    P = unpack(np.asarray(params, dtype=np.float64), table)
    C = {}
    if variant == 2:
        opm, C["opm"] = opm_fwd(P, msa, msa_mask, dims)
        z0 = pair + opm
        m1, m2, m3 = _msa_stack_fwd(P, C, dims, msa, z0, msa_mask, relu_on)
    else:
        m1, m2, m3 = _msa_stack_fwd(P, C, dims, msa, pair, msa_mask, relu_on)
        opm, C["opm"] = opm_fwd(P, m3, msa_mask, dims)
        z0 = pair + opm if variant == 1 else pair
    z1, z2, z3, z4, z5 = _pair_stack_fwd(P, C, dims, z0, pair_mask, relu_on)
    pair_out = z5 + opm if variant == 0 else z5
    inter = dict(m1=m1, m2=m2, m3=m3, opm=opm, z0=z0, z1=z1, z2=z2, z3=z3, z4=z4, z5=z5,
                 mtrans_pre=C["mtrans"][2], ptrans_pre=C["ptrans"][2])
    return m3, pair_out, ((P, C) if want_cache else None), inter


def _msa_stack_bwd(P, G, C, dims, dm):
    dm = dm + transition_bwd(P, G, "mtrans", dm, C["mtrans"])
    if dims["col_global"]:
        dm = dm + col_global_attn_bwd(P, G, dm, C["col"], dims)
    else:
        dm = dm + col_attn_bwd(P, G, dm, C["col"], dims)
    d_row, dz_bias = row_attn_bwd(P, G, dm, C["row"], dims)
    return dm + d_row, dz_bias


def _pair_stack_bwd(P, G, C, dims, dz):
    dz = dz + transition_bwd(P, G, "ptrans", dz, C["ptrans"])
    dz = dz + tri_attn_end_bwd(P, G, "tae", dz, C["tae"], dims)
    dz = dz + tri_attn_start_bwd(P, G, "tas", dz, C["tas"], dims)
    dz = dz + tri_mul_bwd(P, G, "tmi", dz, C["tmi"], False)
    return dz + tri_mul_bwd(P, G, "tmo", dz, C["tmo"], True)


def block_bwd(dims, cache, d_msa_out, d_pair_out):
    """Backward of the block.  Variant 0: as Section "Branch Parallelism" states,
    the cotangent of the block's pair output feeds both the pair stack and the
    outer product mean, and the gradient of the input pair representation is
    the sum of the pair stack's term and the row-attention-bias term.  Variants
    1 and 2 follow from the chain rule on their forward orderings."""
    P, C = cache
    variant = dims.get("variant", 0)
    table, n = param_table(dims)
    G = {}
    if variant == 0:
        dm = d_msa_out + opm_bwd(P, G, d_pair_out, C["opm"], dims)
        dm, dz_bias = _msa_stack_bwd(P, G, C, dims, dm)
        dz = _pair_stack_bwd(P, G, C, dims, d_pair_out)
        d_pair_in = dz + dz_bias
    elif variant == 1:
        dz = _pair_stack_bwd(P, G, C, dims, d_pair_out)          # w.r.t. pair_in + opm
        dm = d_msa_out + opm_bwd(P, G, dz, C["opm"], dims)
        dm, dz_bias = _msa_stack_bwd(P, G, C, dims, dm)
        d_pair_in = dz + dz_bias
    else:
        dz = _pair_stack_bwd(P, G, C, dims, d_pair_out)          # pair stack's share of d(pair_in + opm)
        dm, dz_bias = _msa_stack_bwd(P, G, C, dims, d_msa_out)   # bias was read from pair_in + opm
        d_pair_in = dz + dz_bias
        dm = dm + opm_bwd(P, G, d_pair_in, C["opm"], dims)       # opm read the block's input MSA
    gflat = np.zeros(n)
    for e in table:
        k = int(np.prod(e["shape"]))
        gflat[e["offset"]:e["offset"] + k] = np.asarray(G[e["name"]]).reshape(-1)
    return dm, d_pair_in, gflat, dict(dz_pair_branch=dz, dz_bias=dz_bias)


def block_fwd_bwd(dims, params, msa, pair, msa_mask, pair_mask, d_msa_out, d_pair_out):
    m, z, cache, _ = block_fwd(dims, params, msa, pair, msa_mask, pair_mask)
    dm, dz, g, _ = block_bwd(dims, cache, d_msa_out, d_pair_out)
    return m, z, dm, dz, g


# --------------------------------------------------------------------------
# stack: n_extra extra-MSA blocks then n_main main blocks (Figure 2 caption:
# the extra MSA stack is made of Evoformer blocks; 52 = 48 + 4).  The pair
# representation flows through all blocks; the extra-MSA representation is
# dropped after the extra blocks.
# --------------------------------------------------------------------------
def stack_fwd_bwd(n_extra, dims_e, n_main, dims_m, params, extra_msa, msa, pair,
                  extra_mask, msa_mask, pair_mask, d_msa_out, d_pair_out, recompute=True):
    ne = param_table(dims_e)[1] if n_extra else 0
    nm = param_table(dims_m)[1] if n_main else 0
    saved, caches = [], []
    e, m, z = extra_msa, msa, pair
    off = 0
    for b in range(n_extra + n_main):
        is_e = b < n_extra
        d_, n_ = (dims_e, ne) if is_e else (dims_m, nm)
        x, mk = (e, extra_mask) if is_e else (m, msa_mask)
        saved.append((x, z, off, n_, is_e))
        xo, zo, cache, _ = block_fwd(d_, params[off:off + n_], x, z, mk, pair_mask,
                                     want_cache=not recompute)
        caches.append(cache)
        if is_e:
            e = xo
        else:
            m = xo
        z = zo
        off += n_
    msa_out, pair_out = m, z
    g = np.zeros_like(params)
    dz = d_pair_out
    dm = d_msa_out
    de = np.zeros_like(extra_msa) if n_extra else None
    for b in reversed(range(n_extra + n_main)):
        x, zin, off, n_, is_e = saved[b]
        d_ = dims_e if is_e else dims_m
        mk = extra_mask if is_e else msa_mask
        cache = caches[b]
        if cache is None:
            _, _, cache, _ = block_fwd(d_, params[off:off + n_], x, zin, mk, pair_mask)
        dx, dz, gb, _ = block_bwd(d_, cache, de if is_e else dm, dz)
        g[off:off + n_] = gb
        if is_e:
            de = dx
        else:
            dm = dx
    return msa_out, pair_out, de, dm, dz, g
