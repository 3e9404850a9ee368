"""Transfer orchestrator (include/pipemax_xfer.h) in its host-only mode: the queue discipline against the
model in oracle/xfer_oracle.py (exact issue order), data integrity, and an urgent copy that arrives while a
bulk transfer is in progress."""
import os
import re
import time

import numpy as np
import pytest

from oracle import xfer_oracle as xo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_symbol_of_the_transfer_header(lib):
    hdr = open(os.path.join(ROOT, "include", "pipemax_xfer.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(pipemax_(?:xfer|stage)_[a-z_]+)\s*\(", hdr))
    assert declared == set(lib.XFER_SYMBOLS)
    import ctypes as C
    assert C.sizeof(lib.XferConfig) == 24 and C.sizeof(lib.XferStats) == 80 and C.sizeof(lib.XferLog) == 32


# ---- pins of the model -------------------------------------------------------------------------------
def test_model_hand_example():
    """chunk 4: bulk A (ticket 1, H2D, 10 bytes) -> 4+4+2; urgent (ticket 2, D2H, 3); bulk B (ticket 3, D2H, 5)
    -> 4+1; bulk C (ticket 4, H2D, 4) -> 4.  Urgent first; then the directions alternate, H2D first, each
    direction in arrival order: A0 B0 A1 B1 A2 C0."""
    reqs = [(1, xo.BULK, xo.H2D, 10), (2, xo.URGENT, xo.D2H, 3), (3, xo.BULK, xo.D2H, 5), (4, xo.BULK, xo.H2D, 4)]
    assert xo.issue_order(reqs, 4) == [
        (2, 0, 3, xo.URGENT, xo.D2H),
        (1, 0, 4, xo.BULK, xo.H2D), (3, 0, 4, xo.BULK, xo.D2H),
        (1, 4, 4, xo.BULK, xo.H2D), (3, 4, 1, xo.BULK, xo.D2H),
        (1, 8, 2, xo.BULK, xo.H2D), (4, 0, 4, xo.BULK, xo.H2D)]
    assert xo.chunks_of(0, 4) == [(0, 0)] and xo.chunks_of(9, 0) == [(0, 9)] and xo.chunks_of(8, 4) == [(0, 4), (4, 4)]


@pytest.mark.parametrize("seed", range(4))
def test_model_invariants(seed):
    rng = np.random.default_rng(seed)
    reqs = [(t + 1, int(rng.integers(0, 2)), int(rng.integers(0, 2)), int(rng.integers(0, 50))) for t in range(30)]
    order = xo.issue_order(reqs, 8)
    n_urgent = sum(1 for r in reqs if r[1] == xo.URGENT)
    assert all(e[3] == xo.URGENT for e in order[:n_urgent]) and all(e[3] == xo.BULK for e in order[n_urgent:])
    assert [e[0] for e in order[:n_urgent]] == [r[0] for r in reqs if r[1] == xo.URGENT]
    for t, k, d, n in reqs:                                   # every byte exactly once, in offset order
        parts = [(o, s) for tt, o, s, _, _ in order if tt == t]
        assert [o for o, _ in parts] == sorted(o for o, _ in parts)
        assert sum(s for _, s in parts) == n and all(s <= 8 for _, s in parts if k == xo.BULK)
    for d in (xo.H2D, xo.D2H):                                # a direction serves its requests one after the other
        seq = [e[0] for e in order if e[3] == xo.BULK and e[4] == d]
        assert seq == sorted(seq)


# ---- the library against the model ---------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(5))
def test_issue_order_matches_the_model(lib, seed):
    rng = np.random.default_rng(10 + seed)
    chunk = int(rng.choice([4096, 8192, 65536]))
    x = lib.Xfer(device=-1, max_inflight_bulk=int(rng.integers(1, 4)), chunk_bytes=chunk, log_capacity=4096)
    x.debug_pause(True)
    reqs, bufs = [], []
    for _ in range(int(rng.integers(1, 25))):
        kind, d = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        n = int(rng.choice([0, 1, 100, chunk - 1, chunk, chunk + 1, 3 * chunk + 17]))
        src = rng.integers(0, 256, max(n, 1), dtype=np.uint8)
        dst = np.zeros_like(src)
        t = x.submit(kind, d, dst.ctypes.data, src.ctypes.data, n)
        reqs.append((t, kind, d, n))
        bufs.append((src, dst, n))
    assert [r[0] for r in reqs] == list(range(1, len(reqs) + 1))
    x.debug_pause(False)
    x.drain()
    assert x.log() == xo.issue_order(reqs, chunk)
    for src, dst, n in bufs:
        np.testing.assert_array_equal(dst[:n], src[:n])
    st = x.stats()
    assert st["requests"]["urgent"] + st["requests"]["bulk"] == len(reqs)
    assert st["bytes"]["bulk"] == sum(n for _, k, _, n in reqs if k == xo.BULK)
    assert st["chunks"]["bulk"] == sum(len(xo.chunks_of(n, chunk)) for _, k, _, n in reqs if k == xo.BULK)
    x.destroy()


def test_urgent_copy_overtakes_a_bulk_transfer_in_progress(lib):
    """Sec. 3.4.2: a latency-critical copy that arrives while KV traffic is queued is issued promptly:
    behind at most the chunk being copied, never behind the rest of the bulk request."""
    x = lib.Xfer(device=-1, max_inflight_bulk=1, chunk_bytes=1 << 20, log_capacity=256)
    x.debug_set_host_us_per_mib(3000)                         # 3 ms per chunk, 32 chunks = 96 ms of bulk
    src = np.arange(32 << 20, dtype=np.uint8)
    dst = np.zeros_like(src)
    a, b = np.full(4096, 7, np.uint8), np.zeros(4096, np.uint8)
    t_bulk = x.submit(lib.XFER_BULK, lib.XFER_H2D, dst.ctypes.data, src.ctypes.data, src.nbytes)
    time.sleep(0.010)
    t0 = time.perf_counter()
    t_u = x.submit(lib.XFER_URGENT, lib.XFER_D2H, b.ctypes.data, a.ctypes.data, a.nbytes)
    x.wait(t_u)
    lat = time.perf_counter() - t0
    assert (b == 7).all()
    assert not (dst == src).all()                             # the bulk transfer is still going
    x.wait(t_bulk)
    np.testing.assert_array_equal(dst, src)
    log = x.log()
    pos = [i for i, e in enumerate(log) if e[0] == t_u][0]
    assert 1 <= pos <= 12                                     # some chunks before it, most after
    assert lat < 0.030                                        # about one chunk, not the 60+ ms that were left
    st = x.stats()
    assert st["latency_max_s"]["urgent"] < 0.030 < st["latency_max_s"]["bulk"]
    x.destroy()


def test_argument_and_state_errors(lib):
    x = lib.Xfer(device=-1)
    buf = np.zeros(16, np.uint8)
    for kind, d in ((2, 0), (0, 2), (-1, 0)):
        with pytest.raises(lib.PipemaxError) as e:
            x.submit(kind, d, buf.ctypes.data, buf.ctypes.data, 16)
        assert e.value.code == lib.ERR_ARG
    with pytest.raises(lib.PipemaxError) as e:
        x.submit(lib.XFER_BULK, lib.XFER_H2D, 0, buf.ctypes.data, 16)
    assert e.value.code == lib.ERR_ARG
    for bad in (0, 99):
        with pytest.raises(lib.PipemaxError) as e:
            x.wait(bad)
        assert e.value.code == lib.ERR_ARG
    t = x.submit(lib.XFER_URGENT, lib.XFER_H2D, 0, 0, 0)      # an empty copy completes
    x.wait(t)
    with pytest.raises(lib.PipemaxError) as e:
        x.stream_wait(t, 0)
    assert e.value.code == lib.ERR_STATE
    x.destroy()
    for bad in (dict(max_inflight_bulk=0), dict(chunk_bytes=100), dict(device=-2)):
        with pytest.raises(lib.PipemaxError) as e:
            lib.Xfer(**{**dict(device=-1), **bad})
        assert e.value.code == lib.ERR_ARG
