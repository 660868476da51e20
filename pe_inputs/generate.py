"""Seeded input generator (numpy PCG64).

Draw order: msa, pair, masks, parameters in flat-layout order, then the output
cotangents.  The parameter table (name, offset, shape, fan_in, kind) is passed
in by the caller, so this file knows nothing about the block itself.
"""
import numpy as np


def round_to_bf16(x):
    """Round float values to the nearest bfloat16 (ties to even); returns float64."""
    a = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    u = a.view(np.uint32).astype(np.uint64)
    bias = ((u >> 16) & 1) + 0x7FFF
    u = ((u + bias) >> 16) << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(a.shape)


def res_mask_for(recipe, s, r, rng):
    """Return (msa_mask[s,r], pair_mask[r,r]) of 0/1 float64 for a mask recipe."""
    kind, arg = recipe
    if kind == "none":
        return np.ones((s, r)), np.ones((r, r))
    if kind == "last_residues":
        res = np.ones(r)
        if arg > 0:
            res[-int(arg):] = 0.0
        return np.tile(res, (s, 1)), np.outer(res, res)
    if kind == "first_residues":
        res = np.ones(r)
        res[:int(arg)] = 0.0
        return np.tile(res, (s, 1)), np.outer(res, res)
    if kind == "random_residues":
        n = int(round(arg * r))
        res = np.ones(r)
        res[rng.choice(r, size=n, replace=False)] = 0.0
        return np.tile(res, (s, 1)), np.outer(res, res)
    if kind == "random_rows":
        n = int(round(arg * s))
        rows = np.ones(s)
        rows[rng.choice(s, size=n, replace=False)] = 0.0
        return np.tile(rows[:, None], (1, r)), np.ones((r, r))
    raise ValueError(kind)


def make_params(table, n_params, rng):
    """table: iterable of dicts with offset, shape, fan_in, kind in
    {'weight','ln_gamma','ln_beta','bias'}.  Weights ~ N(0, 1/fan_in);
    LN gains 1 + 0.1 N(0,1); LN offsets and biases 0.1 N(0,1)."""
    p = np.zeros(n_params, dtype=np.float64)
    for e in table:
        n = int(np.prod(e["shape"]))
        z = rng.standard_normal(n)
        if e["kind"] == "weight":
            v = z / np.sqrt(float(e["fan_in"]))
        elif e["kind"] == "ln_gamma":
            v = 1.0 + 0.1 * z
        else:
            v = 0.1 * z
        p[e["offset"]:e["offset"] + n] = v
    return p


def make_inputs(dims, table, n_params, mask_recipe, seed, n_blocks=1, scale=1.0):
    """Returns a dict of float64 arrays.  If dims['dtype'] is bf16 the
    activations and cotangents are pre-rounded to bf16-representable values
    (parameters stay full precision, stored as fp32-representable)."""
    rng = np.random.default_rng(seed)
    s, r, c_m, c_z = dims["s"], dims["r"], dims["c_m"], dims["c_z"]
    msa = scale * rng.standard_normal((s, r, c_m))
    pair = scale * rng.standard_normal((r, r, c_z))
    msa_mask, pair_mask = res_mask_for(mask_recipe, s, r, rng)
    params = np.concatenate([make_params(table, n_params, rng) for _ in range(n_blocks)])
    d_msa_out = rng.standard_normal((s, r, c_m))
    d_pair_out = rng.standard_normal((r, r, c_z))
    params = params.astype(np.float32).astype(np.float64)
    if dims["dtype"] == 1:
        msa, pair = round_to_bf16(msa), round_to_bf16(pair)
        d_msa_out, d_pair_out = round_to_bf16(d_msa_out), round_to_bf16(d_pair_out)
    else:
        f = lambda a: a.astype(np.float32).astype(np.float64)
        msa, pair, d_msa_out, d_pair_out = f(msa), f(pair), f(d_msa_out), f(d_pair_out)
    return dict(msa=msa, pair=pair, msa_mask=msa_mask, pair_mask=pair_mask,
                params=params, d_msa_out=d_msa_out, d_pair_out=d_pair_out)
