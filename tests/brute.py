"""Scalar-loop definitions of every sub-operation of the block (test side).

Written index by index from the definitions, with Python floats and math.exp,
no numpy vector arithmetic.  Used only to pin the vectorised oracle on tiny
inputs.
"""
import math

import numpy as np


def sig(x):
    return 1.0 / (1.0 + math.exp(-x))


def ln_rows(x, g, b, eps):
    x = np.asarray(x)
    out = np.zeros_like(x)
    C = x.shape[-1]
    flat = x.reshape(-1, C)
    of = out.reshape(-1, C)
    for n in range(flat.shape[0]):
        mu = sum(flat[n, c] for c in range(C)) / C
        var = sum((flat[n, c] - mu) ** 2 for c in range(C)) / C
        for c in range(C):
            of[n, c] = (flat[n, c] - mu) / math.sqrt(var + eps) * g[c] + b[c]
    return out


def linear(x, w, b=None):
    x = np.asarray(x)
    K, N = w.shape
    flat = x.reshape(-1, K)
    out = np.zeros((flat.shape[0], N))
    for m in range(flat.shape[0]):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += flat[m, k] * w[k, n]
            out[m, n] = acc + (b[n] if b is not None else 0.0)
    return out.reshape(x.shape[:-1] + (N,))


def attention_one(qrow, keys, vals, blog, kappa, d):
    """One query: weights over valid keys, weighted sum of values."""
    L = len(keys)
    logit = [sum(qrow[t] * keys[j][t] for t in range(d)) / math.sqrt(d) + blog[j] for j in range(L)]
    valid = [j for j in range(L) if kappa[j] > 0]
    out = [0.0] * d
    w = [0.0] * L
    if not valid:
        return out, w
    mx = max(logit[j] for j in valid)
    den = sum(math.exp(logit[j] - mx) for j in valid)
    for j in valid:
        w[j] = math.exp(logit[j] - mx) / den
        for t in range(d):
            out[t] += w[j] * vals[j][t]
    return out, w


def gated_attention(xh, P, pre, H, d, bias, kappa):
    """xh [B,L,c]; bias [H,L,L] or None; kappa [B,L]; returns update [B,L,c]."""
    B, L, c = xh.shape
    q = linear(xh, P[pre + ".w_q"]).reshape(B, L, H, d)
    k = linear(xh, P[pre + ".w_k"]).reshape(B, L, H, d)
    v = linear(xh, P[pre + ".w_v"]).reshape(B, L, H, d)
    g = linear(xh, P[pre + ".w_g"], P[pre + ".b_g"]).reshape(B, L, H, d)
    og = np.zeros((B, L, H, d))
    for b in range(B):
        for h in range(H):
            for i in range(L):
                bl = [bias[h, i, j] if bias is not None else 0.0 for j in range(L)]
                o, _ = attention_one(q[b, i, h], k[b, :, h], v[b, :, h], bl, kappa[b], d)
                for t in range(d):
                    og[b, i, h, t] = sig(g[b, i, h, t]) * o[t]
    return linear(og.reshape(B, L, H * d), P[pre + ".w_o"], P[pre + ".b_o"])


def row_attn(P, m, pair, msa_mask, H, d, eps):
    mh = ln_rows(m, P["row.ln_m.g"], P["row.ln_m.b"], eps)
    zh = ln_rows(pair, P["row.ln_z.g"], P["row.ln_z.b"], eps)
    bz = linear(zh, P["row.w_bias"])            # [r,r,H]
    r = pair.shape[0]
    bias = np.zeros((H, r, r))
    for h in range(H):
        for i in range(r):
            for j in range(r):
                bias[h, i, j] = bz[i, j, h]
    return gated_attention(mh, P, "row", H, d, bias, msa_mask)


def col_attn(P, m, msa_mask, H, d, eps):
    s, r, c = m.shape
    mh = ln_rows(m, P["col.ln.g"], P["col.ln.b"], eps)
    mt = np.zeros((r, s, c))
    kt = np.zeros((r, s))
    for a in range(s):
        for i in range(r):
            mt[i, a] = mh[a, i]
            kt[i, a] = msa_mask[a, i]
    u = gated_attention(mt, P, "col", H, d, None, kt)
    out = np.zeros((s, r, c))
    for a in range(s):
        for i in range(r):
            out[a, i] = u[i, a]
    return out


def col_global_attn(P, m, msa_mask, H, d, eps):
    s, r, c = m.shape
    mh = ln_rows(m, P["col.ln.g"], P["col.ln.b"], eps)
    q = linear(mh, P["col.w_q"]).reshape(s, r, H, d)
    k = linear(mh, P["col.w_k"])
    v = linear(mh, P["col.w_v"])
    g = linear(mh, P["col.w_g"], P["col.b_g"]).reshape(s, r, H, d)
    og = np.zeros((s, r, H, d))
    for i in range(r):
        den = sum(msa_mask[a, i] for a in range(s)) + 1e-10
        for h in range(H):
            qbar = [sum(msa_mask[a, i] * q[a, i, h, t] for a in range(s)) / den for t in range(d)]
            o, _ = attention_one(qbar, k[:, i], v[:, i], [0.0] * s, msa_mask[:, i], d)
            for a in range(s):
                for t in range(d):
                    og[a, i, h, t] = sig(g[a, i, h, t]) * o[t]
    return linear(og.reshape(s, r, H * d), P["col.w_o"], P["col.b_o"])


def tri_attn(P, pre, z, pair_mask, H, d, eps, ending):
    r = z.shape[0]
    zh = ln_rows(z, P[pre + ".ln.g"], P[pre + ".ln.b"], eps)
    q = linear(zh, P[pre + ".w_q"]).reshape(r, r, H, d)
    k = linear(zh, P[pre + ".w_k"]).reshape(r, r, H, d)
    v = linear(zh, P[pre + ".w_v"]).reshape(r, r, H, d)
    g = linear(zh, P[pre + ".w_g"], P[pre + ".b_g"]).reshape(r, r, H, d)
    bz = linear(zh, P[pre + ".w_bias"])          # [r,r,H]
    og = np.zeros((r, r, H, d))
    for i in range(r):
        for j in range(r):
            for h in range(H):
                if not ending:
                    keys = [k[i, kk, h] for kk in range(r)]
                    vals = [v[i, kk, h] for kk in range(r)]
                    bl = [bz[j, kk, h] for kk in range(r)]
                    kap = [pair_mask[i, kk] for kk in range(r)]
                else:
                    keys = [k[kk, j, h] for kk in range(r)]
                    vals = [v[kk, j, h] for kk in range(r)]
                    bl = [bz[kk, i, h] for kk in range(r)]
                    kap = [pair_mask[kk, j] for kk in range(r)]
                o, _ = attention_one(q[i, j, h], keys, vals, bl, kap, d)
                for t in range(d):
                    og[i, j, h, t] = sig(g[i, j, h, t]) * o[t]
    return linear(og.reshape(r, r, H * d), P[pre + ".w_o"], P[pre + ".b_o"])


def transition(P, pre, x, eps):
    xh = ln_rows(x, P[pre + ".ln.g"], P[pre + ".ln.b"], eps)
    a = linear(xh, P[pre + ".w1"], P[pre + ".b1"])
    h = np.zeros_like(a)
    fa, fh = a.reshape(-1), h.reshape(-1)
    for n in range(fa.shape[0]):
        fh[n] = fa[n] if fa[n] > 0 else 0.0
    return linear(h, P[pre + ".w2"], P[pre + ".b2"])


def tri_mul(P, pre, z, pair_mask, eps, outgoing):
    r = z.shape[0]
    zh = ln_rows(z, P[pre + ".ln_in.g"], P[pre + ".ln_in.b"], eps)
    ap = linear(zh, P[pre + ".w_ap"], P[pre + ".b_ap"])
    ag = linear(zh, P[pre + ".w_ag"], P[pre + ".b_ag"])
    bp = linear(zh, P[pre + ".w_bp"], P[pre + ".b_bp"])
    bg = linear(zh, P[pre + ".w_bg"], P[pre + ".b_bg"])
    gr = linear(zh, P[pre + ".w_g"], P[pre + ".b_g"])
    ct = ap.shape[-1]
    a = np.zeros((r, r, ct))
    b = np.zeros((r, r, ct))
    for i in range(r):
        for j in range(r):
            for c in range(ct):
                a[i, j, c] = pair_mask[i, j] * sig(ag[i, j, c]) * ap[i, j, c]
                b[i, j, c] = pair_mask[i, j] * sig(bg[i, j, c]) * bp[i, j, c]
    x = np.zeros((r, r, ct))
    for i in range(r):
        for j in range(r):
            for c in range(ct):
                acc = 0.0
                for k in range(r):
                    acc += a[i, k, c] * b[j, k, c] if outgoing else a[k, i, c] * b[k, j, c]
                x[i, j, c] = acc
    xh = ln_rows(x, P[pre + ".ln_out.g"], P[pre + ".ln_out.b"], eps)
    u = linear(xh, P[pre + ".w_o"], P[pre + ".b_o"])
    out = np.zeros_like(u)
    for i in range(r):
        for j in range(r):
            for c in range(u.shape[-1]):
                out[i, j, c] = sig(gr[i, j, c]) * u[i, j, c]
    return out


def opm(P, m, msa_mask, c_o, eps, eps_o):
    s, r, _ = m.shape
    mh = ln_rows(m, P["opm.ln.g"], P["opm.ln.b"], eps)
    a = linear(mh, P["opm.w_a"], P["opm.b_a"])
    b = linear(mh, P["opm.w_b"], P["opm.b_b"])
    O = np.zeros((r, r, c_o * c_o))
    for i in range(r):
        for j in range(r):
            n = eps_o + sum(msa_mask[t, i] * msa_mask[t, j] for t in range(s))
            for p in range(c_o):
                for q in range(c_o):
                    acc = 0.0
                    for t in range(s):
                        acc += (msa_mask[t, i] * a[t, i, p]) * (msa_mask[t, j] * b[t, j, q])
                    O[i, j, p * c_o + q] = acc / n
    return linear(O, P["opm.w_o"], P["opm.b_o"])


def block(dims, P, msa, pair, msa_mask, pair_mask, variant=0):
    """variant 0: outer product mean of the MSA stack's output added at the end (Figure 1(c));
    1: added to the pair input before the pair stack (Figure 1(a)); 2: outer product mean of the
    INPUT MSA added first, both stacks read the sum (Figure 1(b))."""
    eps = dims["ln_eps"]
    Hm, dm, Hp, dp = dims["h_msa"], dims["d_msa"], dims["h_pair"], dims["d_pair"]
    o_in = opm(P, msa, msa_mask, dims["c_opm"], eps, dims["opm_eps"]) if variant == 2 else None
    bias_pair = pair + o_in if variant == 2 else pair
    m1 = msa + row_attn(P, msa, bias_pair, msa_mask, Hm, dm, eps)
    if dims["col_global"]:
        m2 = m1 + col_global_attn(P, m1, msa_mask, Hm, dm, eps)
    else:
        m2 = m1 + col_attn(P, m1, msa_mask, Hm, dm, eps)
    m3 = m2 + transition(P, "mtrans", m2, eps)
    if variant == 0:
        z0 = pair
    elif variant == 1:
        z0 = pair + opm(P, m3, msa_mask, dims["c_opm"], eps, dims["opm_eps"])
    else:
        z0 = bias_pair
    z1 = z0 + tri_mul(P, "tmo", z0, pair_mask, eps, True)
    z2 = z1 + tri_mul(P, "tmi", z1, pair_mask, eps, False)
    z3 = z2 + tri_attn(P, "tas", z2, pair_mask, Hp, dp, eps, False)
    z4 = z3 + tri_attn(P, "tae", z3, pair_mask, Hp, dp, eps, True)
    z5 = z4 + transition(P, "ptrans", z4, eps)
    if variant == 0:
        return m3, z5 + opm(P, m3, msa_mask, dims["c_opm"], eps, dims["opm_eps"])
    return m3, z5
