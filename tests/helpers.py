"""Shared test helpers (CPU side): seeded inputs through the oracle's table."""
import numpy as np

from oracle.params import param_table, unpack
from pe_inputs import make_inputs, TINY_TEST_DIMS, dims_for


def tiny_case(seed=0, col_global=0, mask=("last_residues", 1), **over):
    dims = dict(TINY_TEST_DIMS)
    dims["col_global"] = col_global
    dims.update(over)
    table, n = param_table(dims)
    inp = make_inputs(dims, table, n, mask, seed)
    return dims, table, n, inp


def named_case(name):
    dims, mask, seed = dims_for(name)
    table, n = param_table(dims)
    return dims, table, n, make_inputs(dims, table, n, mask, seed)


def P_of(inp, table):
    return unpack(inp["params"], table)


def rel_err(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    den = np.max(np.abs(b))
    return float(np.max(np.abs(a - b)) / (den if den > 0 else 1.0))
