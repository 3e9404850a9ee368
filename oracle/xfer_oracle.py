"""Plain model of the transfer orchestrator's queue discipline (lists only).

TEST INFRASTRUCTURE ONLY, like the rest of oracle/.

Passage followed: demand-priority transfer orchestration (Sec. 3.4.2): priorities are enforced through the
order in which copies are submitted; latency-critical (activation) transfers are issued promptly, KV
prefetch and offload opportunistically.  Reading fixed here: urgent requests go out whole, in arrival
order, before any waiting bulk chunk; bulk requests are cut into chunks of at most chunk_bytes; the two
directions take turns, one chunk each, host-to-device first; within a direction requests are served in
arrival order, each to completion.
"""
from __future__ import annotations

URGENT, BULK = 0, 1
H2D, D2H = 0, 1


def chunks_of(nbytes: int, chunk_bytes: int):
    """(offset, size) pieces of one bulk request."""
    if nbytes == 0 or chunk_bytes == 0:
        return [(0, nbytes)]
    return [(o, min(chunk_bytes, nbytes - o)) for o in range(0, nbytes, chunk_bytes)]


def issue_order(requests, chunk_bytes: int):
    """requests: list of (ticket, kind, dir, nbytes), all queued before the dispatcher looks.
    Returns the copies in the order they are handed to the runtime: (ticket, offset, size, kind, dir)."""
    out = [(t, 0, n, URGENT, d) for t, k, d, n in requests if k == URGENT]
    pending = {d: [(t, o, s) for t, k, dd, n in requests if k == BULK and dd == d
                   for o, s in chunks_of(n, chunk_bytes)] for d in (H2D, D2H)}
    while pending[H2D] or pending[D2H]:
        for d in (H2D, D2H):
            if pending[d]:
                t, o, s = pending[d].pop(0)
                out.append((t, o, s, BULK, d))
    return out
