"""CPU tests of the decode-time estimator (Eq. 2) and the prefetch budget (Eq. 6)."""
import numpy as np

from paper_2605_02189_amd import estimator as est


def test_fit_recovers_a_linear_model_exactly():
    rng = np.random.default_rng(0)
    b = rng.integers(1, 65, 40)
    L = b * rng.integers(100, 4000, 40)
    t = 3e-6 * b + 4e-9 * L + 1.1e-3
    m = est.fit(b, L, t)
    assert abs(m.alpha - 3e-6) < 1e-12 and abs(m.beta - 4e-9) < 1e-15 and abs(m.delta - 1.1e-3) < 1e-10
    acc = est.accuracy(m, b, L, t)
    assert acc["within_5pct"] == 1.0 and acc["worst_dev"] < 1e-9


def test_fit_is_least_squares_under_noise():
    rng = np.random.default_rng(1)
    b = rng.integers(1, 65, 400)
    L = b * rng.integers(100, 4000, 400)
    t = (2e-6 * b + 5e-9 * L + 1e-3) * (1 + 0.01 * rng.standard_normal(400))
    m = est.fit(b, L, t)
    assert abs(m.beta / 5e-9 - 1) < 0.02 and abs(m.delta / 1e-3 - 1) < 0.05
    acc = est.accuracy(m, b, L, t)
    assert acc["within_5pct"] > 0.99


def test_budget_is_bandwidth_times_time_and_converts_to_tokens():
    assert est.prefetch_budget_bytes(2e-3, 55e9) == 110e6
    assert est.prefetch_budget_tokens(2e-3, 55e9, 32768) == 110e6 / 32768
    m = est.DecodeTimeModel(0.0, 0.0, 1.5e-3)
    # configs[1]: 64 x 1024 tokens, 32 KiB per token: about 3.8 % of a micro-batch hides behind a step
    s = est.hidden_streamed_fraction(m, 64, 64 * 1024, 55e9, 32768)
    assert abs(s - 1.5e-3 * 55e9 / 32768 / 65536) < 1e-12 and 0.03 < s < 0.05
