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


def test_model_evaluation_goes_through_the_scheduler_and_matches_the_oracle():
    """Eq. 2 and Eq. 6 have one implementation in the product, the scheduler's; the fitted model hands its
    parameters to it.  Values against the scheduler oracle's plain formulas, bit for bit."""
    from oracle import scheduler_oracle as so
    m = est.DecodeTimeModel(2.7e-6, 6.3e-9, 0.87e-3)
    link_tokens_per_s = 56.7e9 / 32768
    sched = m.scheduler(link_tokens_per_s=link_tokens_per_s, n_batches=4)
    for b, L in ((64, 64 * 1024), (1, 0), (128, 300000), (17, 12345)):
        t_hat = sched.predict(b, L)
        assert t_hat == so.predict_time(m.alpha, m.beta, m.delta, b, L)
        assert sched.budget(t_hat) == so.budget_tokens(link_tokens_per_s, t_hat)
    # configs[1]: 64 x 1024 tokens, 32 KiB per token: about 3.8 % of a micro-batch hides behind a step
    s = sched.budget(sched.predict(64, 65536)) / 65536
    assert 0.03 < s < 0.05
    sched.destroy()
