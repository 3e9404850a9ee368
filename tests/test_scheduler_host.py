"""The library's scheduler (C ABI of include/pipemax_sched.h, host code) against the scheduler oracle,
decision by decision.  Bar: identical index lists, counts and flags (integer work); the predicted times
are the same double-precision expression on both sides and must agree to the last bit."""
import os
import re

import numpy as np
import pytest

from oracle import scheduler_oracle as so

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_symbol_of_the_scheduler_header(lib):
    hdr = open(os.path.join(ROOT, "include", "pipemax_sched.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(pipemax_sched_[a-z_]+)\s*\(", hdr))
    assert declared == set(lib.SCHED_SYMBOLS)
    for name in declared:
        assert getattr(lib._lib, name) is not None


def test_struct_sizes_match_the_scheduler_header(lib):
    import ctypes as C
    assert C.sizeof(lib.SchedConfig) == 6 * 8 + 8 + 4 * 4
    assert C.sizeof(lib.SchedIter) == 8 * 4 + 3 * 8 + 2 * 8


def test_create_rejects_bad_configurations(lib):
    ok = dict(alpha_s=1e-6, beta_s=1e-9, delta_s=1e-3, link_tokens_per_s=1e6, n_batches=4)
    lib.Scheduler(**ok).destroy()
    for bad in (dict(window=0), dict(n_batches=0), dict(max_refine_steps=-1), dict(alpha_s=-1.0),
                dict(beta_s=float("nan")), dict(static_budget_tokens=-5), dict(page_tokens=0)):
        with pytest.raises(lib.PipemaxError) as e:
            lib.Scheduler(**{**ok, **bad})
        assert e.value.code == lib.ERR_ARG


def test_time_model_budget_and_steady_flag_match_the_oracle(lib):
    rng = np.random.default_rng(0)
    a, b_, d, B = 2.0e-6, 6.55e-9, 0.939e-3, 1.7e6
    s = lib.Scheduler(alpha_s=a, beta_s=b_, delta_s=d, link_tokens_per_s=B, n_batches=4, window=5,
                      steady_rel_range=0.08)
    det = so.SteadyDetector(5, 0.08)
    level = 1000.0
    for _ in range(200):
        nb, L = int(rng.integers(0, 257)), int(rng.integers(0, 1 << 22))
        t = s.predict(nb, L)
        assert t == so.predict_time(a, b_, d, nb, L)                 # bit for bit
        assert s.budget(t) == so.budget_tokens(B, t)
        level = level * float(rng.uniform(0.9, 1.3)) if level < 50_000 else level * float(rng.uniform(0.97, 1.03))
        assert s.observe(int(level)) == det.observe(int(level))
    assert det.steady
    st = lib.Scheduler(alpha_s=a, beta_s=b_, delta_s=d, link_tokens_per_s=B, n_batches=4, static_budget_tokens=4242)
    assert st.budget(0.5) == 4242 and st.budget(0.0) == 4242


@pytest.mark.parametrize("seed", range(10))
def test_fills_and_partition_match_the_oracle(lib, seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(0, 200))
    # few distinct values -> many ties
    L = (rng.integers(1, 12, n) * 100 if seed % 2 else rng.integers(0, 5000, n)).astype(np.int32).tolist()
    for budget in (0, 1, int(sum(L) * 0.1), int(sum(L) * 0.5), sum(L), sum(L) + 10):
        assert lib.sched_short_first_fill(L, budget) == so.short_first_fill(L, budget)
        assert lib.sched_greedy_fill(L, budget) == so.greedy_fill(L, budget)
    for nb in (1, 2, 3, 4, 7):
        assert lib.sched_partition(L, nb) == so.initial_partition(L, nb)


@pytest.mark.parametrize("seed", range(12))
def test_refinement_matches_the_oracle(lib, seed):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(2, 120))
    L = (rng.integers(1, 9, n) * 64 if seed % 3 == 0 else rng.integers(16, 4096, n)).astype(np.int32).tolist()
    alpha, beta = float(rng.choice([2e-6, 5e-5, 1e-3])), 6.5e-9
    tol = float(rng.choice([0.0, alpha / 2]))
    steps = int(rng.integers(0, 20))
    s = lib.Scheduler(alpha_s=alpha, beta_s=beta, delta_s=0.0, link_tokens_per_s=1.0, n_batches=1,
                      max_refine_steps=steps, refine_tol_s=tol)
    for _ in range(6):
        budget = int(rng.integers(min(L), sum(L)))
        # start from the greedy fill, or from an arbitrary selection within the budget
        if rng.random() < 0.5:
            start = so.greedy_fill(L, budget)
        else:
            start, S = [], 0
            for r in rng.permutation(n).tolist():
                if S + L[r] <= budget and rng.random() < 0.5:
                    start.append(r)
                    S += L[r]
        T0 = alpha * len(start) + beta * sum(L[r] for r in start)
        gap = T0 * float(rng.uniform(0.3, 2.5)) + float(rng.uniform(-1, 1)) * alpha
        want = so.refine(L, start, budget, alpha, beta, gap, steps, tol)
        got = s.refine(L, budget, gap, start)
        assert got == want, (budget, gap, start)


def test_refine_rejects_bad_selections(lib):
    s = lib.Scheduler(alpha_s=1.0, beta_s=0.0, delta_s=0.0, link_tokens_per_s=1.0, n_batches=1)
    for sel, budget in (([0, 0], 100), ([3], 100), ([-1], 100), ([0, 1], 5)):
        with pytest.raises(lib.PipemaxError) as e:
            s.refine([4, 4, 4], budget, 1.0, sel)
        assert e.value.code == lib.ERR_ARG


def _pair(lib, seed, static=0, n=4, b=40, frac=0.55, link=1.7e6, max_len=1500, spare=0.03):
    rng = np.random.default_rng(seed)
    lens = [rng.integers(1, max_len, int(rng.integers(b // 2, b + 1))).tolist() for _ in range(n)]
    resident = [[bool(rng.random() < frac) for _ in l] for l in lens]
    used = sum(-(-lens[k][s] // 16) for k in range(n) for s in range(len(lens[k])) if resident[k][s])
    free = 2 * b + int(spare * used)
    kw = dict(alpha=2e-6, beta=6.55e-9, delta=0.939e-3, link_tokens_per_s=link, window=6, rel_range=0.05,
              max_refine_steps=8, refine_tol=1e-6, static_budget_tokens=static)
    sim = so.SchedulerSim(lens, resident, free, **kw)
    s = lib.Scheduler(alpha_s=kw["alpha"], beta_s=kw["beta"], delta_s=kw["delta"], link_tokens_per_s=link,
                      n_batches=n, window=6, steady_rel_range=0.05, max_refine_steps=8, refine_tol_s=1e-6,
                      static_budget_tokens=static)
    for k in range(n):
        s.set_batch(k, lens[k], [int(r) for r in resident[k]])
    s.set_gpu_pages_free(free)
    return sim, s


@pytest.mark.parametrize("seed,static,n", [(0, 0, 4), (1, 0, 4), (2, 0, 3), (3, 0, 5), (4, 3000, 4), (5, 0, 2),
                                            (6, 0, 1), (7, 40_000, 4)])
def test_alg1_iterations_match_the_oracle_on_the_counted_model(lib, seed, static, n):
    sim, s = _pair(lib, seed, static, n=n, spare=0.03 if n >= 3 else 2.0)   # nothing can be released when n < 3
    saw_steady = saw_exchange = saw_evict = False
    for t in range(120):
        want = sim.iterate(t)
        got = s.plan(t)
        assert got["exec_batch"] == want["exec_batch"] and got["exec"] == want["exec"], t
        assert got["prefetch_batch"] == want["prefetch_batch"] and got["prefetch"] == want["prefetch"], t
        assert got["evict_batch"] == want["evict_batch"] and got["evict"] == want["evict"], t
        assert got["t_hat_s"] == want["t_hat"] and got["gap_s"] == want["d_t"], t
        assert got["budget_tokens"] == want["budget"] and bool(got["steady"]) == want["steady"], t
        assert got["n_exchanges"] == want["exchanges"] and got["gpu_pages_free"] == want["gpu_pages_free"], t
        assert got["prefetch_tokens"] == sum(sim.L[want["prefetch_batch"]][q] for q in want["prefetch"])
        saw_steady |= want["steady"]
        saw_exchange |= want["exchanges"] > 0
        saw_evict |= len(want["evict"]) > 0
    if n >= 3 and not static:
        assert saw_steady and saw_evict


def test_plan_reports_state_errors_and_leaves_the_mirror_unchanged(lib):
    s = lib.Scheduler(alpha_s=1e-6, beta_s=1e-9, delta_s=1e-3, link_tokens_per_s=1e6, n_batches=3)
    with pytest.raises(lib.PipemaxError) as e:
        s.plan(0)                                         # free pages unknown
    assert e.value.code == lib.ERR_STATE
    s.set_gpu_pages_free(0)
    with pytest.raises(lib.PipemaxError) as e:
        s.plan(0)                                         # batches undeclared
    assert e.value.code == lib.ERR_STATE
    for k in range(3):
        s.set_batch(k, [16, 32], [1, 1])                  # both take a new page at the next step
    with pytest.raises(lib.PipemaxError) as e:
        s.plan(0)                                         # no free page for the step
    assert e.value.code == lib.ERR_STATE
    s.set_gpu_pages_free(100)
    d = s.plan(0)
    assert d["exec"] == [0, 1] and d["gpu_pages_free"] == 98
    with pytest.raises(lib.PipemaxError) as e:
        s.plan(-1)
    assert e.value.code == lib.ERR_ARG
    with pytest.raises(lib.PipemaxError):
        s.set_batch(3, [1], [1])
