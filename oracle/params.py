"""Flat parameter layout used by the oracle (TEST INFRASTRUCTURE).

One fp32-valued flat vector per block, the "tensor fusion" the paper describes
(all small parameter tensors fused into one large tensor; Section "Related
Work", fusion paragraph, and Conclusion of "End-to-end training performance").
Weight matrices are row-major [in, out].  The order below is an interface shared
with the C library by specification only: the library has its own table, and a
test compares the two entry by entry.
"""


def _attn(prefix, c_in, h, d, c_bias=None, global_kv=False):
    hd = h * d
    e = [(prefix + ".ln.g", (c_in,), 0, "ln_gamma"), (prefix + ".ln.b", (c_in,), 0, "ln_beta")]
    if c_bias is not None:
        if prefix == "row":
            e = [("row.ln_m.g", (c_in,), 0, "ln_gamma"), ("row.ln_m.b", (c_in,), 0, "ln_beta"),
                 ("row.ln_z.g", (c_bias,), 0, "ln_gamma"), ("row.ln_z.b", (c_bias,), 0, "ln_beta")]
        e.append((prefix + ".w_bias", (c_bias, h), c_bias, "weight"))
    kv = d if global_kv else hd
    e += [(prefix + ".w_q", (c_in, hd), c_in, "weight"),
          (prefix + ".w_k", (c_in, kv), c_in, "weight"),
          (prefix + ".w_v", (c_in, kv), c_in, "weight"),
          (prefix + ".w_g", (c_in, hd), c_in, "weight"),
          (prefix + ".b_g", (hd,), 0, "bias"),
          (prefix + ".w_o", (hd, c_in), hd, "weight"),
          (prefix + ".b_o", (c_in,), 0, "bias")]
    return e


def _trans(prefix, c, n):
    return [(prefix + ".ln.g", (c,), 0, "ln_gamma"), (prefix + ".ln.b", (c,), 0, "ln_beta"),
            (prefix + ".w1", (c, n * c), c, "weight"), (prefix + ".b1", (n * c,), 0, "bias"),
            (prefix + ".w2", (n * c, c), n * c, "weight"), (prefix + ".b2", (c,), 0, "bias")]


def _trimul(prefix, c_z, c_t):
    e = [(prefix + ".ln_in.g", (c_z,), 0, "ln_gamma"), (prefix + ".ln_in.b", (c_z,), 0, "ln_beta")]
    for nm in ("ap", "ag", "bp", "bg"):
        e += [(prefix + ".w_" + nm, (c_z, c_t), c_z, "weight"), (prefix + ".b_" + nm, (c_t,), 0, "bias")]
    e += [(prefix + ".w_g", (c_z, c_z), c_z, "weight"), (prefix + ".b_g", (c_z,), 0, "bias"),
          (prefix + ".ln_out.g", (c_t,), 0, "ln_gamma"), (prefix + ".ln_out.b", (c_t,), 0, "ln_beta"),
          (prefix + ".w_o", (c_t, c_z), c_t, "weight"), (prefix + ".b_o", (c_z,), 0, "bias")]
    return e


def param_table(dims):
    """List of dicts {name, offset, shape, fan_in, kind} in flat order."""
    c_m, c_z = dims["c_m"], dims["c_z"]
    c_o = dims["c_opm"]
    e = []
    e += _attn("row", c_m, dims["h_msa"], dims["d_msa"], c_bias=c_z)
    e += _attn("col", c_m, dims["h_msa"], dims["d_msa"], global_kv=bool(dims["col_global"]))
    e += _trans("mtrans", c_m, dims["n_trans"])
    e += [("opm.ln.g", (c_m,), 0, "ln_gamma"), ("opm.ln.b", (c_m,), 0, "ln_beta"),
          ("opm.w_a", (c_m, c_o), c_m, "weight"), ("opm.b_a", (c_o,), 0, "bias"),
          ("opm.w_b", (c_m, c_o), c_m, "weight"), ("opm.b_b", (c_o,), 0, "bias"),
          ("opm.w_o", (c_o * c_o, c_z), c_o * c_o, "weight"), ("opm.b_o", (c_z,), 0, "bias")]
    e += _trimul("tmo", c_z, dims["c_tri"])
    e += _trimul("tmi", c_z, dims["c_tri"])
    e += _attn("tas", c_z, dims["h_pair"], dims["d_pair"], c_bias=c_z)
    e += _attn("tae", c_z, dims["h_pair"], dims["d_pair"], c_bias=c_z)
    e += _trans("ptrans", c_z, dims["n_trans"])
    out, off = [], 0
    for name, shape, fan_in, kind in e:
        n = 1
        for v in shape:
            n *= v
        out.append(dict(name=name, offset=off, shape=tuple(shape), fan_in=fan_in, kind=kind))
        off += n
    return out, off


def unpack(flat, table):
    """Views of a flat vector as a dict name -> array of the entry's shape."""
    p = {}
    for e in table:
        n = 1
        for v in e["shape"]:
            n *= v
        p[e["name"]] = flat[e["offset"]:e["offset"] + n].reshape(e["shape"])
    return p
