"""GPU-side test helpers: the device harness of the package plus the error metrics of the tests."""
import numpy as np

from paper_2211_00235_amd.harness import BlockRun, tdtype, to_dev, to_np  # noqa: F401


def rel_err(a, b):
    den = np.max(np.abs(b))
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - b)) / (den if den > 0 else 1.0))


def param_errors(g_gpu, g_ref, table):
    """Per-entry max|gpu-ref| / max|ref_entry|.  Entries whose exact gradient is zero
    (row.ln_z.b: a per-head constant added to all logits cancels in the softmax) are
    normalised by the sibling LayerNorm gain's gradient instead."""
    out = {}
    by_name = {e["name"]: e for e in table}
    for e in table:
        n = int(np.prod(e["shape"]))
        sl = slice(e["offset"], e["offset"] + n)
        ref = g_ref[sl]
        den = np.max(np.abs(ref))
        if e["name"] == "row.ln_z.b":
            s = by_name["row.ln_z.g"]
            den = np.max(np.abs(g_ref[s["offset"]:s["offset"] + n]))
        out[e["name"]] = float(np.max(np.abs(g_gpu[sl] - ref)) / (den if den > 0 else 1.0))
    return out
