"""Plain model of the stage's KV bookkeeping (sets, dicts and integers only).

TEST INFRASTRUCTURE ONLY, like the rest of oracle/.  No page arithmetic is
shared with the library: pages here are counted, never addressed.

Passages followed:
  * cyclic batch roles, Eq. 3 (Sec. 3.3.2): at iteration t the stage executes
    D[t mod n], prefetches into D[(i+1) mod n] and may overwrite D[(i-1) mod n];
  * GPU-resident / CPU-resident request sets R_t (Sec. 3.3.2, Alg. 1);
  * the host replica of every sequence is always complete (Sec. 3.4.2,
    asynchronous CPU-assisted offloading), so releasing GPU pages copies nothing;
  * token budget per batch (M - W/n)/T and system capacity (nM - W)/T
    (Eq. 1, App. A.2);
  * KV bytes per token of a stage = 2 * layers * kv_heads * head_dim * elem_bytes.
"""
from __future__ import annotations

HOST, INFLIGHT, GPU = "HOST", "INFLIGHT", "GPU"


def cyclic_roles(t: int, n: int):
    """(execute, prefetch, overwrite) micro-batch indices at iteration t (Eq. 3)."""
    i = t % n
    return i, (i + 1) % n, (i - 1) % n


def kv_bytes_per_token(n_layers: int, n_kv_heads: int, head_dim: int, elem_bytes: int) -> int:
    return 2 * n_layers * n_kv_heads * head_dim * elem_bytes


def token_budget_per_batch(M: float, W: float, n: int, T: float) -> float:
    """Average token budget per decode batch under n-way pipeline parallelism (Eq. 1)."""
    return (M - W / n) / T


def system_token_capacity(M: float, W: float, n: int, T: float) -> float:
    """System-wide maximum number of storable tokens (App. A.2)."""
    return (n * M - W) / T


def pages_for(tokens: int, page_tokens: int) -> int:
    return -(-tokens // page_tokens)


class BookkeepingError(Exception):
    def __init__(self, kind: str):
        super().__init__(kind)
        self.kind = kind


class ResidencyModel:
    """Expected state after each boundary call.

    Per (mb, seq): a context length and one of HOST / INFLIGHT / GPU.
    INFLIGHT = a prefetch has been issued and not yet consumed by a decode
    step; it counts as usable by decode_step (the library orders the work).
    Pool sizes are counted in pages so that exhaustion can be predicted.
    """

    def __init__(self, n_microbatches: int, page_tokens: int, max_ctx: int,
                 gpu_pages: int, host_pages: int, host_reserve_tokens: int = 0):
        self.n = n_microbatches
        self.pt = page_tokens
        self.max_ctx = max_ctx
        self.gpu_free = gpu_pages
        self.host_free = host_pages
        self.reserve = host_reserve_tokens
        self.host_held = {}   # (mb, seq) -> host pages held (in use + reserved)
        self.len = {}      # (mb, seq) -> tokens
        self.state = {}    # (mb, seq) -> HOST | INFLIGHT | GPU
        self.nseq = {}     # mb -> number of sequences

    # -- calls --------------------------------------------------------------
    def mb_define(self, mb: int, ctx_lens):
        if mb in self.nseq or not (0 <= mb < self.n):
            raise BookkeepingError("ARG")
        if any(l < 0 or l > self.max_ctx for l in ctx_lens):
            raise BookkeepingError("ARG")
        held = [pages_for(min(self.max_ctx, l + self.reserve), self.pt) for l in ctx_lens]
        if sum(held) > self.host_free:
            raise BookkeepingError("POOL_EXHAUSTED")
        self.host_free -= sum(held)
        self.nseq[mb] = len(ctx_lens)
        for s, l in enumerate(ctx_lens):
            self.len[(mb, s)] = int(l)
            self.state[(mb, s)] = HOST
            self.host_held[(mb, s)] = held[s]

    def _seqs(self, mb, seq_ids):
        if mb not in self.nseq:
            raise BookkeepingError("ARG")
        if seq_ids is None:
            return list(range(self.nseq[mb]))
        if any(not (0 <= s < self.nseq[mb]) for s in seq_ids):
            raise BookkeepingError("ARG")
        return list(seq_ids)

    def prefetch(self, mb: int, seq_ids=None):
        todo = [s for s in self._seqs(mb, seq_ids) if self.state[(mb, s)] == HOST]
        need = sum(pages_for(self.len[(mb, s)], self.pt) for s in todo)
        if need > self.gpu_free:
            raise BookkeepingError("POOL_EXHAUSTED")
        self.gpu_free -= need
        for s in todo:
            self.state[(mb, s)] = INFLIGHT
        return todo

    def decode_step(self, mb: int):
        seqs = self._seqs(mb, None)
        if any(self.state[(mb, s)] == HOST for s in seqs):
            raise BookkeepingError("NOT_RESIDENT")
        if any(self.len[(mb, s)] + 1 > self.max_ctx for s in seqs):
            raise BookkeepingError("STATE")
        growing = [s for s in seqs if self.len[(mb, s)] % self.pt == 0]
        # a growing sequence first uses a page it holds in reserve, then the pool
        from_pool = [s for s in growing if self.host_held[(mb, s)] <= pages_for(self.len[(mb, s)], self.pt)]
        if len(growing) > self.gpu_free or len(from_pool) > self.host_free:
            raise BookkeepingError("POOL_EXHAUSTED")
        self.gpu_free -= len(growing)
        self.host_free -= len(from_pool)
        for s in from_pool:
            self.host_held[(mb, s)] += 1
        for s in seqs:
            self.len[(mb, s)] += 1
            self.state[(mb, s)] = GPU

    def evict(self, mb: int, seq_ids=None):
        for s in self._seqs(mb, seq_ids):
            if self.state[(mb, s)] != HOST:
                self.gpu_free += pages_for(self.len[(mb, s)], self.pt)
                self.state[(mb, s)] = HOST

    # -- views --------------------------------------------------------------
    def ctx_lens(self, mb: int):
        return [self.len[(mb, s)] for s in range(self.nseq[mb])]

    def n_pages(self, mb: int, seq: int) -> int:
        return pages_for(self.len[(mb, seq)], self.pt)

    def resident(self, mb: int, seq: int) -> bool:
        return self.state[(mb, seq)] != HOST
