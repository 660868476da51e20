"""CPU pin of the ReLU-decision rule used by the bf16 parity tests (tests/parity.py).

The paper trains with fp32 parameters and bf16 intermediate activations (Section "Hyperparameter
setting").  A transition (Section "Evoformer": LayerNorm, Linear x n, ReLU, Linear) evaluated at that
precision computes its pre-activation `a` from bf16 operands, so `a` carries an error of a few 1e-3 of its
rms value and the on/off decision of every element with |a| below that error is not determined.  This file
emulates the storage points of the bf16 path on the CPU (float64 arithmetic, values rounded to bf16 exactly
where the path stores bf16: the residual stream, the LayerNorm output, the weights per use, the hidden
activation and the two hidden cotangents) and pins three facts, none of which uses the HIP path:

  1. size of the pre-activation error: its maximum over the tensor lies inside
     [PREACT_ERR_MAX / 4, PREACT_ERR_MAX] x rms(a) — the constant that bounds the measured band in
     tests/parity.py is neither loose nor tight by more than that factor;
  2. decisions do flip (about 1e-3 of the elements), and only where |a_exact| <= the error;
  3. the flipped decisions alone put the input cotangent and the first weight's gradient outside the
     2e-2 tolerance, while every other rounding source together stays an order of magnitude inside it —
     which is why the parity test evaluates the oracle under the decisions of the path it checks
     (inside the band only) instead of comparing across different decisions.
"""
import numpy as np
import pytest

from pe_inputs import round_to_bf16 as rb
from tests.parity import PREACT_ERR_MAX, TOL, SIZE_FACTORS, size_factor


def transition_emulated(M, C, n, seed, lowp, decisions=None):
    """Transition forward + backward in float64 with (lowp) or without bf16 storage points."""
    rng = np.random.default_rng(seed)
    x = 2.0 * rng.standard_normal((M, C))            # residual stream a few sub-operations into a block
    g = rb(rng.standard_normal((M, C)))              # cotangent of the output
    gam, bet = 1 + 0.1 * rng.standard_normal(C), 0.1 * rng.standard_normal(C)
    W1, b1 = rng.standard_normal((C, n * C)) / np.sqrt(C), 0.1 * rng.standard_normal(n * C)
    W2 = rng.standard_normal((n * C, C)) / np.sqrt(n * C)
    r = rb if lowp else (lambda v: v)
    xin = r(x)
    mu = xin.mean(-1, keepdims=True)
    xc = xin - mu
    rstd = 1.0 / np.sqrt((xc * xc).mean(-1, keepdims=True) + 1e-5)
    xh = xc * rstd
    y = r(xh * gam + bet)
    W1q, W2q = r(W1), r(W2)
    a = y @ W1q + b1
    on = (a > 0) if decisions is None else decisions
    h = r(np.where(on, a, 0.0))
    dh = r((g @ W2q.T) * on)
    dy = r(dh @ W1q.T)
    dxh = dy * gam
    dx = (dxh - dxh.mean(-1, keepdims=True) - xh * (dxh * xh).mean(-1, keepdims=True)) * rstd
    return dict(a=a, on=on, h=h, dW1=y.T @ dh, db1=dh.sum(0), dW2=h.T @ g, dgam=(dy * xh).sum(0), dx=dx)


def _maxrel(a, b):
    return float(np.max(np.abs(a - b)) / np.max(np.abs(b)))


@pytest.mark.parametrize("C,n", [(256, 4), (128, 4), (32, 2)])
def test_preactivation_error_flips_and_their_effect(C, n):
    M = 4096
    exact = transition_emulated(M, C, n, 7, lowp=False)
    low = transition_emulated(M, C, n, 7, lowp=True)
    low_same = transition_emulated(M, C, n, 7, lowp=True, decisions=exact["on"])
    rms = np.sqrt(np.mean(exact["a"] ** 2))
    err = np.abs(low["a"] - exact["a"]) / rms
    flips = low["on"] != exact["on"]
    report = dict(err_rms=float(np.sqrt(np.mean(err ** 2))), err_max=float(err.max()), flip_frac=float(flips.mean()))
    grads = ("dW1", "db1", "dW2", "dgam", "dx")
    with_flips = {k: _maxrel(low[k], exact[k]) for k in grads}
    without = {k: _maxrel(low_same[k], exact[k]) for k in grads}
    print("C=%d n=%d %s\n  own decisions   %s\n  exact decisions %s" % (C, n, report, with_flips, without))
    bound = PREACT_ERR_MAX[1]
    # 1. the constant brackets the emulated error
    assert bound / 4 <= report["err_max"] <= bound, report
    # 2. decisions flip, rarely, and only inside the error
    assert 1e-4 < report["flip_frac"] < 5e-3, report
    assert np.all(np.abs(exact["a"][flips]) / rms <= err[flips])
    # 3. everything but the flips is far inside the tolerance; the flips alone are outside it
    tol = TOL[1]
    assert max(without.values()) < tol / 3, without
    assert with_flips["dx"] > tol and with_flips["dW1"] > tol, with_flips
    # the forward result does not depend on the decisions inside the band beyond the band itself
    assert np.max(np.abs(low["h"] - low_same["h"])) <= 1.01 * err.max() * rms


def test_max_normalised_metric_by_tensor_size():
    """The parity metric is max|error| / max|reference| per tensor.  With the same per-element error, how far into
    its tail does that ratio reach for a tensor of n entries?  Monte Carlo (iid normal reference entries and errors,
    fixed seed): the 99th percentile over tensors, relative to tensors of 65536 entries, must be covered by the
    size factors that the small-shape bf16 tests apply, and those factors must not be looser than 1.35 x needed."""
    rng = np.random.default_rng(5)

    def q99(n, trials):
        g, e = rng.standard_normal((trials, n)), rng.standard_normal((trials, n))
        return float(np.quantile(np.abs(e).max(1) / np.abs(g).max(1), 0.99))
    big = q99(65536, 300)
    lower = 1
    for limit, f in SIZE_FACTORS:
        smallest = max(lower, 16)               # the smallest tensor the bin is used for
        need = q99(smallest, 4000) / big
        print("entries %d..%d: factor %.2f, needed at %d entries %.2f" % (lower, limit, f, smallest, need))
        assert 0.95 * need <= f <= 1.35 * need, (limit, f, need)
        assert size_factor(limit) == f
        lower = limit + 1
    assert size_factor(lower) == 1.0 and q99(lower, 1000) / big < 1.15
