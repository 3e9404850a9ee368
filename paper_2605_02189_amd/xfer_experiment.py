"""Latency of small urgent copies under KV prefetch traffic (demand-priority transfer orchestration, Sec. 3.4.2).
Run:  python -m paper_2605_02189_amd.xfer_experiment

Bulk traffic: the prefetch of one C2 micro-batch (35 runs of 64 MiB host -> device, 2.3 GB), --rounds times, all
queued at the start, plus the per-step KV write-back (2 MiB device -> host every 1.5 ms).  Urgent traffic: one
512 KiB copy in each direction, standing in for the activation exchange with the neighbouring stages, issued
every millisecond and waited for.  Three ways of issuing the same requests:
  fifo          urgent copies go down the same queues as the KV copies (arrival order)
  own_stream    urgent copies on their own streams; KV runs submitted whole and all at once
  orchestrated  KV runs cut into --chunk-mib chunks, at most --inflight submitted per direction; urgent at once
Prints one JSON object: latency of the urgent pair (mean / p99 / max) and the bulk host->device rate per mode.
"""
from __future__ import annotations

import argparse
import json
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--rounds", type=int, default=3)
    ap.add_argument("--chunk-mib", type=float, default=4.0)
    ap.add_argument("--inflight", type=int, default=2)
    ap.add_argument("--urgent-kib", type=int, default=512)
    ap.add_argument("--sweep", action="store_true", help="also try other chunk sizes and windows")
    args = ap.parse_args()
    import torch
    from . import binding as pm

    run_bytes, n_runs = 64 << 20, 35
    h_kv = torch.empty(n_runs * run_bytes, dtype=torch.uint8).pin_memory()
    h_kv.fill_(1)
    d_kv = torch.empty(n_runs * run_bytes, dtype=torch.uint8, device="cuda:0")
    wb_d = torch.ones(2 << 20, dtype=torch.uint8, device="cuda:0")
    wb_h = torch.empty(2 << 20, dtype=torch.uint8).pin_memory()
    ub = args.urgent_kib << 10
    u_h, u_d = torch.ones(ub, dtype=torch.uint8).pin_memory(), torch.empty(ub, dtype=torch.uint8, device="cuda:0")
    v_d, v_h = torch.ones(ub, dtype=torch.uint8, device="cuda:0"), torch.empty(ub, dtype=torch.uint8).pin_memory()
    torch.cuda.synchronize()

    def run(mode: str, chunk_mib: float = args.chunk_mib, inflight: int = args.inflight) -> dict:
        if mode == "orchestrated":
            x = pm.Xfer(device=0, max_inflight_bulk=inflight, chunk_bytes=int(chunk_mib * (1 << 20)))
        else:
            x = pm.Xfer(device=0, max_inflight_bulk=1 << 20, chunk_bytes=0)
        ukind = pm.XFER_BULK if mode == "fifo" else pm.XFER_URGENT
        t_start = time.perf_counter()
        last = 0
        for _ in range(args.rounds):
            for r in range(n_runs):
                last = x.submit(pm.XFER_BULK, pm.XFER_H2D, d_kv.data_ptr() + r * run_bytes,
                                h_kv.data_ptr() + r * run_bytes, run_bytes)
        lats = []
        next_u = next_wb = t_start + 1.0e-3
        t_done = None
        while time.perf_counter() - t_start < 20.0:
            now = time.perf_counter()
            if t_done is None and x.poll(last):
                t_done = now
                break
            if now >= next_wb:
                x.submit(pm.XFER_BULK, pm.XFER_D2H, wb_h.data_ptr(), wb_d.data_ptr(), wb_h.numel())
                next_wb = now + 1.5e-3
            if now >= next_u:
                t0 = time.perf_counter()
                a = x.submit(ukind, pm.XFER_H2D, u_d.data_ptr(), u_h.data_ptr(), ub)
                b = x.submit(ukind, pm.XFER_D2H, v_h.data_ptr(), v_d.data_ptr(), ub)
                x.wait(a)
                x.wait(b)
                lats.append(time.perf_counter() - t0)
                next_u = time.perf_counter() + 1.0e-3
        x.drain()
        if t_done is None:
            t_done = time.perf_counter()
        x.destroy()
        a = np.array(lats) * 1e3
        return {"bulk_h2d_gbs": args.rounds * n_runs * run_bytes / (t_done - t_start) / 1e9,
                "urgent_pairs": int(a.size), "urgent_ms_mean": float(a.mean()), "urgent_ms_median": float(np.median(a)),
                "urgent_ms_p99": float(np.percentile(a, 99)), "urgent_ms_max": float(a.max())}

    res = {"rounds": args.rounds, "chunk_mib": args.chunk_mib, "inflight": args.inflight,
           "urgent_kib": args.urgent_kib, "modes": {}}
    run("orchestrated")                                       # warm-up: first touches, stream creation
    for mode in ("fifo", "own_stream", "orchestrated"):
        res["modes"][mode] = run(mode)
    if args.sweep:
        res["sweep"] = {}
        for c in (2.0, 4.0, 8.0, 16.0, 32.0):
            for w in (1, 2, 3):
                res["sweep"][f"chunk{c:g}_inflight{w}"] = run("orchestrated", c, w)
    # the same pair with no other traffic
    x = pm.Xfer(device=0)
    idle = []
    for _ in range(200):
        t0 = time.perf_counter()
        a = x.submit(pm.XFER_URGENT, pm.XFER_H2D, u_d.data_ptr(), u_h.data_ptr(), ub)
        b = x.submit(pm.XFER_URGENT, pm.XFER_D2H, v_h.data_ptr(), v_d.data_ptr(), ub)
        x.wait(a)
        x.wait(b)
        idle.append(time.perf_counter() - t0)
    x.destroy()
    res["idle_link_urgent_ms_median"] = float(np.median(idle) * 1e3)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
