"""Candidate-count policy by Equation 1 (Section 1): the library's host functions against the oracle's
written-out definition and against what the formula fixes by itself (CPU only)."""
import math

import numpy as np
import pytest

from oracle import metrics
from paper_2505_08600_amd import api


def test_oracle_equation_1_closed_forms():
    """Pins of the oracle's formula that do not come from the oracle: gamma = 0 is plain decoding
    (speed-up 1 whatever alpha and c), alpha = 0 leaves one token per step, alpha = 1 gives gamma + 1
    tokens, and the numerator is the finite geometric sum."""
    for c in (0.0, 0.03, 0.5):
        for a in (0.0, 0.3, 0.9, 1.0):
            assert metrics.eq1_speedup(a, 0, c) == pytest.approx(1.0)
        for g in (1, 5, 15):
            assert metrics.eq1_speedup(0.0, g, c) == pytest.approx(1.0 / (g * c + 1.0))
            assert metrics.eq1_speedup(1.0, g, c) == pytest.approx((g + 1.0) / (g * c + 1.0))
            assert metrics.eq1_speedup(0.7, g, c) == pytest.approx(sum(0.7 ** i for i in range(g + 1)) / (g * c + 1.0))


def test_oracle_best_gamma_properties():
    """One candidate beats none exactly when alpha > c ((1 + alpha) / (1 + c) > 1); the best count never
    falls when alpha rises or c falls; a free draft (c = 0) with alpha > 0 always wants the maximum."""
    for a in np.linspace(0.0, 1.0, 21):
        for c in (0.01, 0.05, 0.2, 0.6):
            assert (metrics.best_gamma(a, c, 1) == 1) == (a > c + 1e-12)
    for c in (0.01, 0.03, 0.1, 0.3):
        best = [metrics.best_gamma(a, c, 15) for a in np.linspace(0.0, 1.0, 101)]
        assert all(x <= y for x, y in zip(best, best[1:]))
    for a in (0.2, 0.5, 0.8, 0.95):
        best = [metrics.best_gamma(a, c, 15) for c in np.linspace(0.0, 1.0, 101)]
        assert all(x >= y for x, y in zip(best, best[1:]))
        assert metrics.best_gamma(a, 0.0, 15) == 15


def test_library_equation_1_and_choice_match_the_oracle():
    for a in np.linspace(0.0, 1.0, 41):
        for c in (0.0, 0.005, 0.0289, 0.1, 0.35, 1.0, 2.0):
            for g in range(0, 16):
                assert api.eq1_speedup(float(a), g, c) == pytest.approx(metrics.eq1_speedup(float(a), g, c), rel=1e-12)
            for gmax in (0, 1, 5, 10, 15):
                g_lib, v_lib = api.choose_gamma(float(a), c, gmax)
                g_ref = metrics.best_gamma(float(a), c, gmax)
                v_ref = metrics.eq1_speedup(float(a), g_ref, c)
                # (an exact tie between two counts may be broken differently by rounding: the values decide)
                assert v_lib == pytest.approx(v_ref, rel=1e-12)
                assert g_lib == g_ref or metrics.eq1_speedup(float(a), g_lib, c) == pytest.approx(v_ref, rel=1e-12)


def test_library_alpha_hat_matches_the_oracle_and_its_definition():
    rng = np.random.default_rng(5)
    for gamma in (1, 4, 5, 8, 15):
        n_acc = rng.integers(0, gamma + 1, size=200).tolist()
        assert api.alpha_hat(n_acc, gamma) == pytest.approx(metrics.alpha_hat(n_acc, gamma), rel=1e-12)
    # every candidate accepted: alpha = 1; first candidate always rejected: alpha = 0
    assert api.alpha_hat([5, 5, 5], 5) == 1.0 and api.alpha_hat([0, 0], 5) == 0.0
    # geometric acceptance with probability p: the estimate converges to p
    p, gamma = 0.6, 8
    steps = [min(int(rng.geometric(1 - p)) - 1, gamma) for _ in range(200000)]
    assert api.alpha_hat(steps, gamma) == pytest.approx(p, abs=5e-3)
    assert math.isnan(api.alpha_hat([6], 5)) and math.isnan(api.alpha_hat([-1], 5))


def test_library_policy_argument_errors():
    assert math.isnan(api.eq1_speedup(1.5, 3, 0.1)) and math.isnan(api.eq1_speedup(0.5, -1, 0.1))
    assert math.isnan(api.eq1_speedup(0.5, 3, -0.1))
    for bad in ((-0.1, 0.1, 5), (0.5, -1.0, 5), (0.5, 0.1, 16), (0.5, 0.1, -1), (float("nan"), 0.1, 5)):
        with pytest.raises(api.SdError):
            api.choose_gamma(*bad)
