"""The comparison helper of the GPU parity tests does bind (CPU only): results a broken kernel would
give are rejected against oracle values of realistic size and spread."""
import json
import os
import numpy as np
import pytest

from tolerance import check_kl_cases, bound, tight, north_star

RNG = np.random.default_rng(0)
WANT = np.abs(RNG.standard_normal(40)) * 0.3 + 0.01          # KLs of O(0.01 .. 1)
SIGMA = np.where(RNG.random(40) < 0.2, 2e-4, 0.0)            # a few cases with a code move nearby


def test_exact_and_rounding_level_results_pass():
    check_kl_cases(WANT, WANT, SIGMA)
    check_kl_cases(WANT * (1 + 3e-6), WANT, SIGMA)
    k = int(np.argmax(SIGMA))
    flip = WANT.copy(); flip[k] += 4 * SIGMA[k]                   # a case with a code move nearby, moved by four sigma
    check_kl_cases(flip, WANT, SIGMA)


@pytest.mark.parametrize("broken", [
    lambda w: np.zeros_like(w),                 # a kernel that returns 0 for every edge
    lambda w: w * 0.987,                        # every KL 1.3 % low (a truncating adder)
    lambda w: w * 1.01,
    lambda w: w + 5e-3,                         # an offset
    lambda w: np.roll(w, 1),                    # results of the wrong candidates
    lambda w: np.where(np.arange(w.size) == 7, np.nan, w),
])
def test_broken_results_fail(broken):
    with pytest.raises(AssertionError):
        check_kl_cases(broken(WANT), WANT, SIGMA)


def test_one_outlier_beyond_its_spread_fails_and_small_values_bind():
    bad = WANT.copy(); bad[5] *= 1.05
    with pytest.raises(AssertionError):
        check_kl_cases(bad, WANT, np.zeros_like(WANT))
    small = np.full(10, 2e-5)                   # below the benchmark's absolute floor of 1e-4
    assert (north_star(small) > small).all() and (tight(small) < 0.1 * small).all()
    with pytest.raises(AssertionError):
        check_kl_cases(np.zeros(10), small, np.zeros(10))


def test_stored_expected_values_are_large_enough_to_bind():
    """Every golden set marked 'hi' has a median KL that the relative part of the bound governs."""
    gdir = os.path.join(os.path.dirname(__file__), "golden")
    seen = 0
    for f in sorted(os.listdir(gdir)):
        if not (f.startswith("kl_") and ("_hi." in f or "_hi2." in f)):
            continue
        gold = json.load(open(os.path.join(gdir, f)))
        kls = np.array([k for c in gold["cases"] for k in c["kl_new"]])
        assert np.median(kls) >= 2e-3, (f, np.median(kls))        # where 1e-3 |KL| exceeds the 1e-6 floor
        seen += 1
    assert seen >= 1
