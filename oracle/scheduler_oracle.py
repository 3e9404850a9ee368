"""Plain model of the prefetch-aware decode scheduler (lists, sets and Python numbers only).

TEST INFRASTRUCTURE ONLY, like the rest of oracle/.  Nothing here is shared with the library's
scheduler; the two are compared decision by decision in tests/.

Passages followed:
  * decode-time model  alpha*b + beta*L + delta  (Sec. 3.3.1, Eq. 2);
  * prefetch budget  B * T_hat  of the executing batch (Sec. 3.3.2, Eq. 6), counted in cached tokens
    because the selection compares it with prefix lengths (App. A.4, Alg. 2);
  * retained set D_j^res, remaining time gap  dT = T_hat - T_hat_res  (Sec. 3.3.2, Eq. 7);
  * warm-up phase: short requests first, to pack as many requests as the budget allows; steady phase:
    length-first greedy fill followed by exchanges that trade one long request for several short ones
    (or back) until the modelled time of the prefetched set is close to dT (App. A.4, Alg. 1 and 2);
  * steady phase detected when the budgets of the last w iterations vary by less than a threshold,
    relative to their mean (App. A.4);
  * initial partition into n batches of equal size with balanced total length (Sec. 3.3.2).

Choices the paper leaves open (each is a stated reading, not a result):
  * every order is total: by length, ties by request index;
  * one exchange moves exactly one request against two (the pair with the largest total length that
    still fits the budget; the longest replacement that fits), and is applied only if it brings the
    modelled time closer to dT; the first selected request (longest first), respectively the first
    adjacent pair of selected requests (shortest first), that admits such an exchange is taken;
  * the steady flag latches;
  * the partition deals the requests, longest first, to the batches in serpentine order;
  * the candidates of an iteration are the host-resident requests of the batch being updated; the
    requests of the overwritten batch are released oldest-resident first, and only as many as the
    prefetch and the next step's new pages need.
"""
from __future__ import annotations

import math


# ---- Eq. 2, Eq. 6 ----------------------------------------------------------------------------
def predict_time(alpha: float, beta: float, delta: float, b: int, L: int) -> float:
    return alpha * b + beta * L + delta


def budget_tokens(link_tokens_per_s: float, t_hat: float) -> int:
    return int(math.floor(link_tokens_per_s * t_hat))


# ---- steady-phase detection --------------------------------------------------------------------
class SteadyDetector:
    def __init__(self, window: int, rel_range: float):
        self.w, self.thr = window, rel_range
        self.hist = []
        self.steady = False

    def observe(self, budget: int) -> bool:
        self.hist.append(budget)
        recent = self.hist[-self.w:]
        if not self.steady and len(recent) == self.w:
            mean = sum(recent) / self.w
            if mean > 0 and (max(recent) - min(recent)) / mean < self.thr:
                self.steady = True
        return self.steady


# ---- selections ----------------------------------------------------------------------------------
def short_first_fill(L, budget):
    """Warm-up selection: shortest first while the cumulative length stays within the budget."""
    sel, S = [], 0
    for r in sorted(range(len(L)), key=lambda r: (L[r], r)):
        if S + L[r] > budget:
            break
        sel.append(r)
        S += L[r]
    return sel


def greedy_fill(L, budget):
    """Length-first pass of Alg. 2: longest first, every request that still fits is taken."""
    sel, S = [], 0
    for r in sorted(range(len(L)), key=lambda r: (-L[r], r)):
        if S + L[r] <= budget:
            sel.append(r)
            S += L[r]
    return sel


def _by_length_desc(ids, L):
    return sorted(ids, key=lambda r: (-L[r], r))


def _exchange_up(L, sel, budget):
    """Candidate exchanges that add one request: for each selected r, longest first, the pair of
    unselected requests shorter than r with the largest total length that fits."""
    S = sum(L[r] for r in sel)
    for r in _by_length_desc(sel, L):
        cap = budget - (S - L[r])
        pool = _by_length_desc([u for u in range(len(L)) if u not in sel and L[u] < L[r]], L)
        best = None
        for x in range(len(pool)):
            for y in range(x + 1, len(pool)):
                tot = L[pool[x]] + L[pool[y]]
                if tot <= cap and (best is None or tot > best[0]):
                    best = (tot, pool[x], pool[y])
        if best is not None:
            yield r, (best[1], best[2])


def _exchange_down(L, sel, budget):
    """Candidate exchanges that remove one request: for each adjacent pair of selected requests,
    shortest first, the longest unselected request longer than both that fits."""
    S = sum(L[r] for r in sel)
    asc = sorted(sel, key=lambda r: (L[r], r))
    for a, b in zip(asc, asc[1:]):
        cap = budget - (S - L[a] - L[b])
        pool = _by_length_desc([u for u in range(len(L)) if u not in sel and L[b] < L[u] <= cap], L)
        if pool:
            yield (a, b), pool[0]


def refine(L, sel, budget, alpha, beta, d_t, max_steps, tol):
    """Exchange pass of Alg. 2 from a given selection.  Returns (selection, exchanges applied)."""
    sel = list(sel)
    n_ex = 0
    for _ in range(max_steps):
        S = sum(L[r] for r in sel)
        mis = (alpha * len(sel) + beta * S) - d_t
        if abs(mis) <= tol:
            break
        applied = False
        if mis < 0:
            for r, (u, v) in _exchange_up(L, sel, budget):
                S2 = S - L[r] + L[u] + L[v]
                if abs((alpha * (len(sel) + 1) + beta * S2) - d_t) < abs(mis):
                    sel = [x for x in sel if x != r] + [u, v]
                    applied = True
                    break
        else:
            for (a, b), u in _exchange_down(L, sel, budget):
                S2 = S - L[a] - L[b] + L[u]
                if abs((alpha * (len(sel) - 1) + beta * S2) - d_t) < abs(mis):
                    sel = [x for x in sel if x not in (a, b)] + [u]
                    applied = True
                    break
        if not applied:
            break
        n_ex += 1
    return sel, n_ex


def greedy_select(L, budget, alpha, beta, d_t, max_steps, tol):
    """Alg. 2: length-first fill, then the exchange pass."""
    return refine(L, greedy_fill(L, budget), budget, alpha, beta, d_t, max_steps, tol)


# ---- initial partition -----------------------------------------------------------------------------
def initial_partition(L, n):
    """batch_of[r]: requests dealt longest first, forwards then backwards over the n batches."""
    batch_of = [0] * len(L)
    for pos, r in enumerate(_by_length_desc(range(len(L)), L)):
        rnd, k = divmod(pos, n)
        batch_of[r] = k if rnd % 2 == 0 else n - 1 - k
    return batch_of


# ---- Alg. 1 on a counted model of the stage ---------------------------------------------------------
def _pages(tokens, pt):
    return -(-tokens // pt)


class SchedulerSim:
    """Alg. 1 driving a counted model of the stage: per (batch, request) a length, a residency bit
    and the iteration since which it has been resident; GPU pages are counted, never addressed.

    lens[k][s]: prefix lengths; resident[k][s]: True if on the GPU at the start.
    """

    def __init__(self, lens, resident, gpu_pages_free, *, alpha, beta, delta, link_tokens_per_s,
                 window, rel_range, max_refine_steps, refine_tol, static_budget_tokens=0, page_tokens=16):
        self.n = len(lens)
        self.L = [list(map(int, l)) for l in lens]
        self.res = [list(map(bool, r)) for r in resident]
        self.since = [[-1 if x else None for x in r] for r in self.res]
        self.free = int(gpu_pages_free)
        self.a, self.b_, self.d = alpha, beta, delta
        self.B = link_tokens_per_s
        self.det = SteadyDetector(window, rel_range)
        self.max_steps, self.tol = max_refine_steps, refine_tol
        self.static = int(static_budget_tokens)
        self.pt = page_tokens

    def _time(self, k, ids):
        return predict_time(self.a, self.b_, self.d, len(ids), sum(self.L[k][s] for s in ids))

    def iterate(self, t):
        n, pt = self.n, self.pt
        i, j, k = t % n, (t + 1) % n, (t - 1) % n
        E = [s for s in range(len(self.L[i])) if self.res[i][s]]
        t_hat = self._time(i, E)
        budget = self.static if self.static > 0 else budget_tokens(self.B, t_hat)
        steady = self.det.observe(budget)
        # the executing batch takes its new pages first, then grows by one token
        grow_E = sum(1 for s in E if self.L[i][s] % pt == 0)
        assert grow_E <= self.free, "the previous iteration did not leave room for this step's new pages"
        self.free -= grow_E
        for s in E:
            self.L[i][s] += 1
        P, evicted, n_ex, d_t = [], [], 0, 0.0
        if j != i:
            res_j = [s for s in range(len(self.L[j])) if self.res[j][s]]
            cand = [s for s in range(len(self.L[j])) if not self.res[j][s]]
            d_t = t_hat - self._time(j, res_j)
            Lc = [self.L[j][s] for s in cand]
            if steady:
                pick, n_ex = greedy_select(Lc, budget, self.a, self.b_, d_t, self.max_steps, self.tol)
            else:
                pick = short_first_fill(Lc, budget)
            P = [cand[x] for x in pick]

            def need(P_):
                nxt = res_j + P_
                return (sum(_pages(self.L[j][s], pt) for s in P_)
                        + sum(1 for s in nxt if self.L[j][s] % pt == 0))
            if k != i and k != j:
                order = sorted((s for s in range(len(self.L[k])) if self.res[k][s]),
                               key=lambda s: (self.since[k][s], s))
                for s in order:
                    if self.free >= need(P):
                        break
                    self.free += _pages(self.L[k][s], pt)
                    self.res[k][s] = False
                    self.since[k][s] = None
                    evicted.append(s)
            while P and self.free < need(P):
                P.pop()
            assert self.free >= need(P), "no room for the next step's new pages"
            for s in P:
                self.free -= _pages(self.L[j][s], pt)
                self.res[j][s] = True
                self.since[j][s] = t
        return {"exec_batch": i, "exec": E, "prefetch_batch": j, "prefetch": P, "evict_batch": k,
                "evict": evicted, "t_hat": t_hat, "budget": budget, "steady": steady, "d_t": d_t,
                "exchanges": n_ex, "gpu_pages_free": self.free}
