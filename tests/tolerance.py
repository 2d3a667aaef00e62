"""The parity bounds of the GPU tests, stated once.

north_star(kl)   |d| <= 1e-4 + 1e-3 |KL|: the tolerance the benchmark spec fixes for per-edge KL.  Asserted on the
                 five named configurations as they are specified (weights N(0, 0.02)).
bound(kl, s)     |d| <= 1e-6 + 1e-3 |KL| + 5 s: the same relative part, an absolute floor a hundred times
                 lower, and five standard deviations of what binary32 arithmetic leaves undetermined in
                 this value (s: tests/fp32_spread.py, measured on the oracle itself).  Where no quantiser
                 decision is close to a rounding boundary s is 0 and the bound is the tight one; where one
                 is, no binary32 implementation can do better than s.  s is never taken below the rms of
                 the workload's own cases (a rare code move shows in few seeded re-evaluations of one case
                 but in the pool of all of them).
median rule      over the cases of a workload the median of |d| / (1e-6 + 1e-3 |KL| + s) stays below 1: the
                 typical case lies within ONE standard deviation of its spread (on the small shapes, where
                 code moves are the exception and s is 0 for most cases, within the tight bound itself), so
                 a systematic error (a wrong scale, a biased sum, a result of zero) cannot hide behind the
                 five-sigma term that covers the tails.
Increments (kl_new - kl_current, the number ACDC decides on) are held to the same bound with |KL| the
larger of the two values and s the spread of the increment itself.
"""
import numpy as np

KL_ATOL, KL_RTOL = 1e-4, 1e-3
TIGHT_ATOL = 1e-6
SIGMAS = 5.0


def north_star(kl):
    return KL_ATOL + KL_RTOL * np.abs(kl)


def tight(kl):
    return TIGHT_ATOL + KL_RTOL * np.abs(kl)


def bound(kl, sigma):
    return tight(kl) + SIGMAS * np.asarray(sigma, dtype=np.float64)


def pooled(sigma):
    s = np.asarray(sigma, dtype=np.float64)
    return float(np.sqrt(np.mean(s * s))) if s.size else 0.0


def check_median(got, want, what=""):
    """The median rule alone (for sets of cases whose spread has not been measured)."""
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    med = float(np.median(np.abs(got - want) / tight(want)))
    assert med <= 1.0, (what, "median |d| / (1e-6 + 1e-3 |KL|) =", med)
    return med


def check_kl_cases(got, want, sigma, what="", median_rule=True, kl_scale=None):
    """Asserts the bound for every case and the median rule for the set.  kl_scale: the |KL| that sets
    the relative part when it is not |want| itself (increments).  Returns the worst |d| / bound."""
    got, want = np.asarray(got, dtype=np.float64), np.asarray(want, dtype=np.float64)
    sigma = np.asarray(sigma, dtype=np.float64)
    assert got.shape == want.shape == sigma.shape and got.size > 0, what
    assert np.isfinite(got).all(), (what, "non-finite device value")
    scale = np.abs(want) if kl_scale is None else np.asarray(kl_scale, dtype=np.float64)
    s = np.maximum(sigma, pooled(sigma))
    d = np.abs(got - want)
    b = bound(scale, s)
    worst = int(np.argmax(d / b))
    assert (d <= b).all(), (what, "case", worst, "got", got[worst], "want", want[worst], "bound", b[worst])
    if median_rule and got.size >= 8:
        med = float(np.median(d / (tight(scale) + s)))
        assert med <= 1.0, (what, "median |d| / (1e-6 + 1e-3 |KL| + sigma) =", med)
    return float((d / b).max())
