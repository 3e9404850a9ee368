"""Prefill throughput of one stage on this GPU.  Run:
    python -m paper_2605_02189_amd.prefill_bench [--config C2] [--tokens 2048] [--chunk 256] [--requests 4]

Every request is a fresh sequence of --tokens synthetic tokens, fed to pipemax_prefill in chunks of --chunk rows
(the stage's max_seqs_per_mb); the K,V of every layer goes to the GPU pages and, through the write-back stream
and the host re-layout worker, to the pinned host replica (Sec. 3.1.1, Sec. 3.4.2).  Prints one JSON object:
tokens/s, achieved matrix-core rate on the model's FLOPs, per-kernel-class times and the offload rate.
"""
from __future__ import annotations

import argparse
import json
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="C2")
    ap.add_argument("--tokens", type=int, default=2048)
    ap.add_argument("--chunk", type=int, default=256)
    ap.add_argument("--requests", type=int, default=4)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-writeback", action="store_true")
    args = ap.parse_args()
    import torch
    from . import binding as pm
    from .harness import StageRunner
    from .synth_inputs import CONFIGS, SynthInputs

    base = CONFIGS[args.config]
    R, T = args.requests + 1, args.tokens                         # one extra request warms the kernels up
    shape = base.with_(n_microbatches=1, seqs_per_mb=R)
    syn = SynthInputs(shape, seed=args.seed)
    ctx = {0: np.zeros(R, dtype=np.int32)}
    flags = pm.FLAG_NO_WRITEBACK if args.no_writeback else 0
    run = StageRunner(shape, syn, sigma=0.0, steps=T + 16, ctx_lens=ctx, flags=flags,
                      gpu_pages=R * (T // 16 + 2) + 8, max_rows=args.chunk)    # row capacity of a pass = --chunk
    st = run.stage
    run.load_weights()
    st.mb_define(0, ctx[0])
    st.prefetch_kv(0)
    stream = torch.cuda.Stream()
    x = syn.hidden(0, min(T, 4096))
    reps = -(-T // x.shape[0])
    hin = torch.from_numpy(np.tile(x.view(np.int16), (reps, 1))[:T].copy()).view(torch.bfloat16).to("cuda:0")
    hout = torch.empty_like(hin)

    def prefill(seq):
        st.prefill(0, seq, T, hin.data_ptr(), hout.data_ptr(), stream.cuda_stream)

    prefill(0)
    st.sync()
    res = {}
    for timed in (False, True):
        st.set_flags(set_=pm.FLAG_TIME_KERNELS if timed else 0, clear=0 if timed else pm.FLAG_TIME_KERNELS)
        st.reset_stats()
        if not timed:
            first, last = 1, 1 + max(1, args.requests // 2)
        else:
            first, last = 1 + max(1, args.requests // 2), R
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for seq in range(first, last):
            prefill(seq)
        st.sync()
        dt = time.perf_counter() - t0
        n = (last - first) * T
        s = st.get_stats()
        if not timed:
            res["tokens_per_s"] = n / dt
            res["ms_per_request"] = dt / (last - first) * 1e3
            res["d2h_gbs"] = s["d2h_bytes"] / dt / 1e9
            res["requests_timed"] = last - first
            res["host_wait_ms_per_request"] = s["host_wait_s"] / (last - first) * 1e3
            res["host_enqueue_ms_per_request"] = s["host_enqueue_s"] / (last - first) * 1e3
        else:
            res["kernel_ms_per_request"] = {k: round(v / (last - first), 3) for k, v in s["kernel_ms"].items() if v > 0}
            res["kernel_launches_per_request"] = {k: v // (last - first) for k, v in s["kernel_launches"].items() if v}
    h, nq, F = base.hidden, base.n_q_heads * base.head_dim, base.ffn
    nqkv = (base.n_q_heads + 2 * base.n_kv_heads) * base.head_dim
    gemm_flops = 2.0 * (h * nqkv + nq * h + h * 2 * F + F * h) * T * base.n_layers
    attn_flops = 4.0 * base.head_dim * base.n_q_heads * (T * (T + 1) / 2) * base.n_layers
    sec = res["ms_per_request"] * 1e-3
    km = res["kernel_ms_per_request"]
    gemm_ms = sum(km.get(k, 0.0) for k in ("gemm_qkv", "gemm_o", "gemm_gu", "gemm_d"))
    res.update({"config": base.name, "tokens": T, "chunk": args.chunk, "layers": base.n_layers,
                "gemm_tflop": gemm_flops / 1e12, "attn_tflop_causal": attn_flops / 1e12,
                "tflops_end_to_end": (gemm_flops + attn_flops) / sec / 1e12,
                "gemm_tflops_in_kernels": gemm_flops / (gemm_ms * 1e-3) / 1e12 if gemm_ms else None,
                "attn_tflops_in_kernels": attn_flops / (km.get("attn", 0) * 1e-3) / 1e12 if km.get("attn") else None})
    print(json.dumps(res))
    st.destroy()


if __name__ == "__main__":
    main()
