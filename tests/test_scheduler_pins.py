"""Pins of the scheduler oracle (oracle/scheduler_oracle.py) against things other than itself:
brute force over all subsets, hand-worked examples whose arithmetic is written out here, closed forms
and invariants of Alg. 1 / Alg. 2 (App. A.4), Eq. 2 and Eq. 6."""
import itertools

import numpy as np
import pytest

from oracle import scheduler_oracle as so


# ---- Eq. 2, Eq. 6 ------------------------------------------------------------------------------
def test_time_model_and_budget_closed_forms():
    # 2 us per request, 5 ns per token, 1 ms constant: 64 requests of 1024 tokens
    t = so.predict_time(2e-6, 5e-9, 1e-3, 64, 64 * 1024)
    assert t == pytest.approx(64 * 2e-6 + 65536 * 5e-9 + 1e-3, rel=1e-15)
    # linear in b and L separately
    assert so.predict_time(3.0, 0.0, 0.0, 7, 100) == 21.0
    assert so.predict_time(0.0, 0.5, 0.0, 7, 100) == 50.0
    assert so.predict_time(0.0, 0.0, 4.0, 7, 100) == 4.0
    # budget: tokens the link moves in t_hat, rounded down (never more than fits behind the step)
    assert so.budget_tokens(1000.0, 1.5) == 1500
    assert so.budget_tokens(1000.0, 0.0019) == 1
    assert so.budget_tokens(1000.0, 0.0009) == 0


# ---- warm-up selection -----------------------------------------------------------------------------
def _all_subsets(n):
    for k in range(n + 1):
        yield from itertools.combinations(range(n), k)


@pytest.mark.parametrize("seed", range(6))
def test_short_first_fill_packs_the_most_requests_the_budget_allows(seed):
    """Sec. 3.3.2 (warm-up): short requests first maximise the batch size under a KV budget.  Brute force:
    no subset within the budget has more members, and none with as many members is shorter in total."""
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 11))
    L = rng.integers(1, 40, n).tolist()
    budget = int(rng.integers(0, sum(L) + 5))
    sel = so.short_first_fill(L, budget)
    assert len(set(sel)) == len(sel)
    S = sum(L[r] for r in sel)
    assert S <= budget
    best_count = max(len(c) for c in _all_subsets(n) if sum(L[r] for r in c) <= budget)
    assert len(sel) == best_count
    assert S == min(sum(L[r] for r in c) for c in _all_subsets(n)
                    if len(c) == best_count and sum(L[r] for r in c) <= budget)


def test_short_first_fill_hand_example_and_ties():
    # lengths 5 1 3 2, budget 6: ascending 1 (idx1), 2 (idx3), 3 (idx2) -> 6; 5 does not fit
    assert so.short_first_fill([5, 1, 3, 2], 6) == [1, 3, 2]
    # equal lengths are taken in index order
    assert so.short_first_fill([4, 4, 4], 9) == [0, 1]
    assert so.short_first_fill([4, 4, 4], 3) == []
    assert so.short_first_fill([], 10) == []
    assert so.short_first_fill([0, 0], 0) == [0, 1]


# ---- greedy initialisation ---------------------------------------------------------------------------
def test_greedy_fill_hand_examples():
    # budget 9: 5, then 4 (9); 3 and 2 no longer fit
    assert so.greedy_fill([5, 4, 3, 2], 9) == [0, 1]
    # budget 8: 5, 4 does not fit (9 > 8), 3 fits (8), 2 does not
    assert so.greedy_fill([5, 4, 3, 2], 8) == [0, 2]
    # equal lengths: floor(budget / L) of them, lowest indices
    assert so.greedy_fill([7] * 5, 30) == [0, 1, 2, 3]
    assert so.greedy_fill([7] * 5, 6) == []


@pytest.mark.parametrize("seed", range(6))
def test_greedy_fill_stays_within_the_budget_and_is_maximal(seed):
    rng = np.random.default_rng(100 + seed)
    L = rng.integers(1, 300, int(rng.integers(1, 40))).tolist()
    budget = int(rng.integers(0, sum(L)))
    sel = so.greedy_fill(L, budget)
    S = sum(L[r] for r in sel)
    assert S <= budget and len(set(sel)) == len(sel)
    # maximal: nothing left out fits into the slack
    assert all(L[r] > budget - S for r in range(len(L)) if r not in sel)
    # length-first: the selection is in non-increasing length order
    assert [L[r] for r in sel] == sorted((L[r] for r in sel), reverse=True)


# ---- exchange refinement ---------------------------------------------------------------------------------
def test_refinement_hand_example_one_long_request_against_two_short_ones():
    """alpha = 1, beta = 0.01.  Lengths 10 6 5 4 3, budget 10, gap 2.1.
    Greedy: {10}, S = 10, T = 1*1 + 0.01*10 = 1.1 < 2.1.  Exchange: remove 10 (cap = 10); pairs of shorter
    unselected requests within 10: 6+4 = 10, 6+3 = 9, 5+4 = 9, 5+3 = 8, 4+3 = 7 -> (6, 4) = indices (1, 3);
    T' = 2 + 0.1 = 2.1: mismatch 0, applied, and the next pass stops on the tolerance."""
    sel, n_ex = so.greedy_select([10, 6, 5, 4, 3], 10, 1.0, 0.01, 2.1, 8, 1e-9)
    assert (sel, n_ex) == ([1, 3], 1)


def test_refinement_hand_example_two_short_requests_against_one_long_one():
    """alpha = 1, beta = 0.01.  Lengths 2 2 5, selection {0, 1}, budget 6, gap 1.05.
    T = 2 + 0.04 = 2.04 > 1.05.  The two shortest selected (2, 2) leave cap = 6 - 0 = 6; the longest
    unselected request longer than both and within 6 is 5 (index 2); T' = 1 + 0.05 = 1.05: applied."""
    assert so.refine([2, 2, 5], [0, 1], 6, 1.0, 0.01, 1.05, 8, 1e-9) == ([2], 1)


def test_refinement_rejects_exchanges_that_do_not_improve_and_respects_the_step_cap():
    # gap already met within the tolerance: nothing happens
    assert so.refine([10, 6, 4], [0], 10, 1.0, 0.0, 1.2, 8, 0.25) == ([0], 0)
    # the only possible exchange (10 -> 6 + 4) would move T from 1 to 2 with gap 1.4: |0.6| > |0.4|, rejected
    assert so.refine([10, 6, 4], [0], 10, 1.0, 0.0, 1.4, 8, 0.0) == ([0], 0)
    # with gap 1.6 it is accepted (|0.4| < |0.6|)
    assert so.refine([10, 6, 4], [0], 10, 1.0, 0.0, 1.6, 8, 0.0) == ([1, 2], 1)
    # step cap: lengths 8 4 4 2 2 2 2, gap asks for many requests; each step adds exactly one
    L = [8, 4, 4, 2, 2, 2, 2]
    full, n_full = so.refine(L, [0], 8, 1.0, 0.0, 4.0, 8, 0.0)
    assert n_full == 3 and sorted(L[r] for r in full) == [2, 2, 2, 2]
    one, n_one = so.refine(L, [0], 8, 1.0, 0.0, 4.0, 1, 0.0)
    assert n_one == 1 and sorted(L[r] for r in one) == [4, 4]


@pytest.mark.parametrize("seed", range(8))
def test_refinement_invariants_on_random_instances(seed):
    """Alg. 2: the budget is never exceeded, members stay distinct, every exchange changes the count by
    exactly one, and the mismatch to the gap never grows."""
    rng = np.random.default_rng(200 + seed)
    n = int(rng.integers(2, 60))
    L = rng.integers(16, 4096, n).tolist()
    budget = int(rng.integers(min(L), sum(L) // 2 + min(L)))
    alpha, beta = 2e-6, 6.5e-9
    start = so.greedy_fill(L, budget)
    T0 = alpha * len(start) + beta * sum(L[r] for r in start)
    gap = T0 * float(rng.uniform(0.6, 1.6))
    prev_mis, prev_sel = abs(T0 - gap), start
    for steps in range(1, 12):
        sel, n_ex = so.refine(L, start, budget, alpha, beta, gap, steps, 0.0)
        assert len(set(sel)) == len(sel) and sum(L[r] for r in sel) <= budget
        assert n_ex <= steps
        mis = abs(alpha * len(sel) + beta * sum(L[r] for r in sel) - gap)
        assert mis <= prev_mis
        assert abs(len(sel) - len(prev_sel)) <= 1
        if n_ex < steps:
            break
        prev_mis, prev_sel = mis, sel


# ---- steady-phase detection ----------------------------------------------------------------------------
def test_steady_detector_hand_example_and_latch():
    """w = 3, threshold 0.1.  Budgets 100 200 300 310 305: windows (100,200,300): 200/200 = 1.0;
    (200,300,310): 110/270 = 0.41; (300,310,305): 10/305 = 0.033 < 0.1 -> steady at the 5th budget."""
    d = so.SteadyDetector(3, 0.1)
    assert [d.observe(b) for b in (100, 200, 300, 310, 305)] == [False, False, False, False, True]
    assert d.observe(10_000) is True                      # latched
    # a constant budget is steady exactly when the window is full
    d = so.SteadyDetector(4, 0.05)
    assert [d.observe(777) for _ in range(5)] == [False, False, False, True, True]
    # geometric growth by 1.5x never settles: (max - min)/mean of 3 terms = 1.25/1.583 = 0.79
    d = so.SteadyDetector(3, 0.5)
    assert not any(d.observe(int(100 * 1.5 ** k)) for k in range(20))
    # all-zero budgets are not a steady phase
    d = so.SteadyDetector(2, 0.5)
    assert [d.observe(0) for _ in range(3)] == [False, False, False]


# ---- initial partition -----------------------------------------------------------------------------------
def test_partition_hand_example():
    # 9 8 7 | 6 5 4 dealt 0 1 2 | 2 1 0: totals 9+4, 8+5, 7+6 = 13 each
    assert so.initial_partition([9, 8, 7, 6, 5, 4], 3) == [0, 1, 2, 2, 1, 0]
    assert so.initial_partition([5, 5, 5, 5], 2) == [0, 1, 1, 0]
    assert so.initial_partition([], 3) == []
    assert so.initial_partition([3, 1, 2], 1) == [0, 0, 0]


@pytest.mark.parametrize("seed", range(6))
def test_partition_is_equal_sized_and_balanced(seed):
    """Sec. 3.3.2: equal batch sizes, total lengths balanced.  Every request lands in exactly one batch,
    sizes differ by at most one, and (for full double rounds) the heaviest and the lightest batch differ by
    at most the longest request."""
    rng = np.random.default_rng(300 + seed)
    n = int(rng.integers(2, 7))
    N = 2 * n * int(rng.integers(1, 12))
    L = rng.integers(1, 4096, N).tolist()
    part = so.initial_partition(L, n)
    sizes = [part.count(k) for k in range(n)]
    assert sum(sizes) == N and max(sizes) - min(sizes) == 0
    totals = [sum(L[r] for r in range(N) if part[r] == k) for k in range(n)]
    assert max(totals) - min(totals) <= max(L)
    # ragged count: sizes differ by at most one
    part = so.initial_partition(L[: N - 1], n)
    sizes = [part.count(k) for k in range(n)]
    assert max(sizes) - min(sizes) <= 1


# ---- Alg. 1 on the counted stage model -----------------------------------------------------------------------
def _make_sim(seed, static=0, n=4, b=24, frac_resident=0.6, link=2.0e6):
    rng = np.random.default_rng(seed)
    lens = [rng.integers(16, 1500, b).tolist() for _ in range(n)]
    resident = [[bool(rng.random() < frac_resident) for _ in range(b)] for _ in range(n)]
    used = sum(-(-lens[k][s] // 16) for k in range(n) for s in range(b) if resident[k][s])
    free = 2 * b + int(0.05 * used)
    sim = so.SchedulerSim(lens, resident, free, alpha=2e-6, beta=6.5e-9, delta=9e-4, link_tokens_per_s=link,
                          window=6, rel_range=0.05, max_refine_steps=8, refine_tol=1e-6,
                          static_budget_tokens=static)
    return sim, used + free


@pytest.mark.parametrize("seed,static", [(0, 0), (1, 0), (2, 0), (3, 5000)])
def test_alg1_invariants_on_the_counted_model(seed, static):
    sim, total_pages = _make_sim(seed, static)
    n = sim.n
    was_steady = False
    for t in range(60):
        before_res = [list(r) for r in sim.res]
        before_len = [list(l) for l in sim.L]
        d = sim.iterate(t)
        i, j, k = t % n, (t + 1) % n, (t - 1) % n
        assert (d["exec_batch"], d["prefetch_batch"], d["evict_batch"]) == (i, j, k)          # Eq. 3
        # the executed batch is exactly the resident part of D_i; each member grew by one token
        assert d["exec"] == [s for s, r in enumerate(before_res[i]) if r]
        assert all(sim.L[i][s] == before_len[i][s] + 1 for s in d["exec"])
        # Eq. 2 / Eq. 6 on the executed batch
        t_hat = 2e-6 * len(d["exec"]) + 6.5e-9 * sum(before_len[i][s] for s in d["exec"]) + 9e-4
        assert d["t_hat"] == pytest.approx(t_hat, rel=1e-12)
        assert d["budget"] == (static if static else int(2.0e6 * d["t_hat"]))
        # P_t: host-resident requests of D_j, within the budget
        assert all(not before_res[j][s] for s in d["prefetch"])
        assert sum(sim.L[j][s] for s in d["prefetch"]) <= d["budget"]
        assert all(sim.res[j][s] for s in d["prefetch"])
        # released requests were resident members of D_k, and nothing else lost residency
        assert all(before_res[k][s] and not sim.res[k][s] for s in d["evict"])
        for m in range(n):
            for s in range(len(sim.L[m])):
                if before_res[m][s] and not sim.res[m][s]:
                    assert m == k and s in d["evict"]
        # pages are conserved: free + pages of resident requests = pool size
        held = sum(-(-sim.L[m][s] // 16) for m in range(n) for s in range(len(sim.L[m])) if sim.res[m][s])
        assert d["gpu_pages_free"] >= 0 and d["gpu_pages_free"] + held == total_pages
        # the flag latches
        assert d["steady"] or not was_steady
        was_steady = d["steady"]
        if not d["steady"]:
            assert d["exchanges"] == 0
    assert was_steady                                       # the budgets settle within 60 iterations


def test_alg1_warm_up_feeds_back_into_the_budget():
    """Sec. 3.3.2: while there is room, prefetching more requests makes the batches larger, the predicted
    time longer and the next budgets larger."""
    n, b = 3, 40
    lens = [[64] * b for _ in range(n)]
    resident = [[s < 4 for s in range(b)] for _ in range(n)]
    sim = so.SchedulerSim(lens, resident, 10_000, alpha=1e-4, beta=1e-7, delta=1e-3, link_tokens_per_s=3.0e5,
                          window=4, rel_range=0.01, max_refine_steps=4, refine_tol=0.0)
    budgets = [sim.iterate(t)["budget"] for t in range(12)]
    assert all(b2 >= b1 for b1, b2 in zip(budgets, budgets[1:]))
    assert budgets[-1] > budgets[0]
