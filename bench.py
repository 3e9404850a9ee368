#!/usr/bin/env python3
"""Benchmark of the stage-decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C2] [--sigma 1.0]

A step = one pass of the whole hot path over one micro-batch: pipemax_decode_step of D_i with the
KV prefetch of D_{i+1} and the write-back running on the side streams (cyclic schedule, Eq. 3).
The default workload is configs[1] (8 of 32 layers of an 8B-shaped model, 4 micro-batches x 64
sequences x 1024-token prompts, bf16) with every inactive micro-batch's KV in pinned host memory
(sigma = 1).  Inputs (weights, hidden states, the active micro-batch's pages once prefetched) are
resident in HBM when the timed region starts; the KV of the inactive micro-batches is in host
memory by construction: moving it is the method being measured, not input staging.

Prints ONE JSON line.  Besides the headline (tokens/s of the streamed schedule) it carries
  roofline      achieved HBM GB/s of the attention kernel from HIP events on the compute stream,
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload,
  legs          compute-only / transfers-only / both, the overlap fraction and the link rate.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
LINK_PEAK_GBS = 64.0           # PCIe Gen5 x16, one direction (the figure the paper uses, Sec. 4.1)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def attn_bytes(shape, lens_before):
    """Algorithmic bytes of one attention launch: K and V of L_i + 1 tokens, all KV heads, one layer."""
    return sum(2 * shape.n_kv_heads * shape.head_dim * shape.elem_bytes * (int(L) + 1) for L in lens_before)


def measured_traffic(config_name, key="traffic_bytes_per_launch"):
    """HBM bytes per attention launch from the committed rocprofv3 --pmc summary of this workload (and, with
    key="algorithmic_bytes_per_launch", the algorithmic bytes of the launches those counters were read on)."""
    path = os.path.join(ROOT, "profiles", f"attn_{config_name}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith(key):
                return int(line.split()[1])
    except OSError:
        pass
    return None


def cpu_baseline(shape, syn, ctx0, k_seqs, n_steps):
    """The oracle as it stands on a sample of micro-batch 0: k sequences, all layers, full context."""
    import numpy as np
    from oracle.stage_oracle import StageOracle
    orc = StageOracle(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                      shape.ffn, shape.rope_base, shape.rms_eps)
    for l in range(shape.n_layers):
        orc.set_layer_weights(l, **{k: syn.as_f32(v) for k, v in syn.weights(l).items()})
    seqs = list(range(k_seqs))
    for s in seqs:
        kv = [syn.kv_prefix(0, s, l, int(ctx0[0][s])) for l in range(shape.n_layers)]
        orc.define_sequence(0, s, [syn.as_f32(k) for k, _ in kv], [syn.as_f32(v) for _, v in kv])
    x = syn.as_f32(syn.hidden(0, shape.seqs_per_mb))[seqs]
    orc.decode_step(0, x, seqs=seqs)                      # untimed first step (page-in, BLAS start-up)
    t0 = time.perf_counter()
    for _ in range(n_steps):
        orc.decode_step(0, x, seqs=seqs)
    dt = time.perf_counter() - t0
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    try:
        from threadpoolctl import threadpool_info
        blas = [p.get("num_threads") for p in threadpool_info() if p.get("user_api") == "blas"]
        if blas:
            cores = min(cores, max(blas))
    except Exception:
        pass
    return {"value": k_seqs * n_steps / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n_steps} decode steps of {k_seqs} of the {shape.seqs_per_mb} sequences of "
                      f"micro-batch 0, all {shape.n_layers} layers, full {int(ctx0[0][0])}-token context, fp32"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", default="C2")
    ap.add_argument("--sigma", type=float, default=1.0, help="streamed fraction of every micro-batch")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--microbatches", type=int, default=None,
                    help="run with fewer micro-batches than the configuration names (host memory limits)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-legs", action="store_true", help="skip the compute-only / transfer-only legs")
    ap.add_argument("--no-writeback", action="store_true", help="diagnostic: skip the KV write-back (invalid as a result)")
    ap.add_argument("--probe-copy", action="store_true",
                    help="also launch the library's plain copy kernel (256 MiB, 3 times): calibration for --pmc runs")
    ap.add_argument("--sweep", action="store_true",
                    help="also time sigma = 1, 1/2, ..., 1/128, 0 (two cycles each) to locate the crossover "
                         "from link-bound to HBM-bound")
    ap.add_argument("--orchestrated", type=float, default=0.0, metavar="CHUNK_MIB",
                    help="issue the prefetch copies through the transfer orchestrator in chunks of this many MiB "
                         "(window of 2); 0 = the stage's own prefetch stream")
    ap.add_argument("--cpu-seqs", type=int, default=16)
    ap.add_argument("--cpu-steps", type=int, default=48)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one pipeline stage on ONE GPU; --gpus must be 1 "
              "(the stages of a pipeline are independent processes, one per GPU; nothing here runs on a second GPU)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2605_02189_amd.build import ensure_built
    ensure_built()      # loads what is built; builds only if nothing is
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.harness import StageRunner
    from paper_2605_02189_amd.synth_inputs import CONFIGS, SynthInputs

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    shape = CONFIGS[args.config]
    if args.microbatches:
        shape = shape.with_(n_microbatches=args.microbatches)
    n = shape.n_microbatches
    K = args.steps if args.steps is not None else shape.decode_steps
    W = args.warmup if args.warmup is not None else 2 * n
    legs_steps = 0 if args.no_legs else (W + 3 * min(K, 16 * n))
    total_steps = (W + K) + legs_steps + 4 * n + (9 * 4 * n if args.sweep else 0)

    t_setup = time.perf_counter()
    syn = SynthInputs(shape, seed=args.seed)
    run = StageRunner(shape, syn, sigma=args.sigma, steps=total_steps, gpu_pool_all_resident=not args.no_legs,
                      flags=pm.FLAG_NO_WRITEBACK if args.no_writeback else 0)
    st = run.stage
    run.load()
    xfer = None
    if args.orchestrated > 0:
        xfer = pm.Xfer(device=0, max_inflight_bulk=2, chunk_bytes=int(args.orchestrated * (1 << 20)))
        st.attach_xfer(xfer)
    hin = [run.hidden_tensor(mb, mb) for mb in range(n)]
    hout = [torch.empty_like(h) for h in hin]
    stream = torch.cuda.current_stream()
    log(f"setup {time.perf_counter() - t_setup:.1f}s: {shape.name} engine={st.get_stats()['engine']} "
        f"weights {shape.weight_bytes / 1e9:.2f} GB, KV/mb {sum(int(l) for l in run.ctx0[0]) * shape.kv_bytes_per_token / 1e9:.2f} GB")

    def sync():
        torch.cuda.synchronize()
        st.sync()

    legs = {}
    roofline = None
    # ---- the timed run: compute + transfers, the literal configuration -----------------------------------
    run.warm_start()
    for _ in range(W):
        i = run.t % n
        run.step(hin[i], hout[i], stream)
    sync()
    st.reset_stats()
    t0 = time.perf_counter()
    for _ in range(K):
        i = run.t % n
        run.step(hin[i], hout[i], stream)
    sync()
    dt = time.perf_counter() - t0
    s3 = st.get_stats()
    tokens = s3["tokens"]
    value = tokens / dt
    ms_per_step = dt / K * 1e3
    if not args.no_legs:
        # ---- leg 1: compute only (everything resident), kernel classes timed with HIP events -----------
        for mb in range(n):
            st.prefetch_kv(mb)
        sync()
        for _ in range(W):
            i = run.t % n
            run.step(hin[i], hout[i], stream, transfers=False)
        sync()
        Kc = min(K, 16 * n)
        # (a) only the attention kernel bracketed by HIP events on the compute stream: the roofline figure
        st.set_flags(pm.FLAG_TIME_KERNELS | pm.FLAG_TIME_ATTN_ONLY, 0)
        st.reset_stats()
        bytes_attn = 0
        for _ in range(Kc):
            i = run.t % n
            bytes_attn += shape.n_layers * attn_bytes(shape, st.get_ctx_lens(i))
            run.step(hin[i], hout[i], stream, transfers=False)
        sync()
        s0 = st.get_stats()
        attn_ms = s0["kernel_ms"]["attn"] / max(s0["kernel_launches"]["attn"], 1)
        attn_launches = int(s0["kernel_launches"]["attn"])
        # (b) every kernel class bracketed: the per-class breakdown (the brackets themselves cost time)
        st.set_flags(pm.FLAG_TIME_KERNELS, pm.FLAG_TIME_ATTN_ONLY)
        st.reset_stats()
        t0 = time.perf_counter()
        for _ in range(Kc):
            i = run.t % n
            run.step(hin[i], hout[i], stream, transfers=False)
        sync()
        t_timed = time.perf_counter() - t0
        s1 = st.get_stats()
        st.set_flags(0, pm.FLAG_TIME_KERNELS)
        # (c) the same steps without any bracket: the compute-only step time
        t0 = time.perf_counter()
        for _ in range(Kc):
            i = run.t % n
            run.step(hin[i], hout[i], stream, transfers=False)
        sync()
        t_c = (time.perf_counter() - t0) / Kc
        kms, kl = s1["kernel_ms"], s1["kernel_launches"]
        achieved = bytes_attn / max(attn_launches, 1) / (attn_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "k_attn (GQA paged decode attention, split-K pass)",
                    "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(shape.name),
                    "traffic_measured_on_algorithmic_bytes": measured_traffic(shape.name, "algorithmic_bytes_per_launch"),
                    "avg_launch_us": round(attn_ms * 1e3, 2), "launches": attn_launches,
                    "bytes_per_launch": int(bytes_attn / max(attn_launches, 1))}
        hbm_bytes_step = shape.weight_bytes + bytes_attn / Kc
        legs["compute_only"] = {
            "ms_per_step": round(t_c * 1e3, 4), "tokens_per_s": round(run.b / t_c, 1),
            "ms_per_step_with_event_brackets": round(t_timed / Kc * 1e3, 4),
            "hbm_bytes_per_step": int(hbm_bytes_step),
            "frac_of_hbm_roofline": round(hbm_bytes_step / t_c / 1e9 / HBM_PEAK_GBS, 4),
            "kernel_us_per_launch": {k: round(kms[k] / max(kl[k], 1) * 1e3, 2) for k in kms if kl[k]},
            "kernel_ms_per_step": {k: round(kms[k] / Kc, 4) for k in kms if kl[k]},
            "gemm_tflops": round(2 * (shape.weight_bytes / shape.elem_bytes) * run.b /
                                 ((kms["gemm_qkv"] + kms["gemm_o"] + kms["gemm_gu"] + kms["gemm_d"]) / Kc * 1e-3) / 1e12, 1),
            "gemm_weight_gbs": round(shape.weight_bytes /
                                     ((kms["gemm_qkv"] + kms["gemm_o"] + kms["gemm_gu"] + kms["gemm_d"]) / Kc * 1e-3) / 1e9, 1),
            "host_enqueue_ms_per_step": round(s1["host_enqueue_s"] / Kc * 1e3, 4)}
        log("compute-only:", json.dumps(legs["compute_only"]))
        # ---- leg 2: transfers only (the same evict / prefetch traffic, no kernels) ---------------------
        for mb in range(n):
            st.evict_kv(mb)
        sync()
        run.t = 0
        run.warm_start()
        sync()
        st.set_flags(pm.FLAG_TIME_KERNELS, 0)
        st.reset_stats()
        Kx = 2 * n
        t0 = time.perf_counter()
        for _ in range(Kx):
            run.step(None, None, stream, compute=False)
        sync()
        t_x = (time.perf_counter() - t0) / Kx
        s2 = st.get_stats()
        st.set_flags(0, pm.FLAG_TIME_KERNELS)
        legs["transfer_only"] = {
            "ms_per_step": round(t_x * 1e3, 3), "h2d_bytes_per_step": int(s2["h2d_bytes"] / Kx),
            "h2d_copies_per_step": s2["h2d_copies"] / Kx,
            "h2d_gbs_busy": round(s2["h2d_bytes"] / max(s2["h2d_ms"], 1e-9) / 1e6, 2),
            "h2d_gbs_wall": round(s2["h2d_bytes"] / Kx / t_x / 1e9, 2)}
        log("transfer-only:", json.dumps(legs["transfer_only"]))
        for mb in range(n):
            st.evict_kv(mb)
        sync()
        run.t = 0

    if legs:
        t_both = dt / K
        t_c, t_x = legs["compute_only"]["ms_per_step"] * 1e-3, legs["transfer_only"]["ms_per_step"] * 1e-3
        legs["both"] = {
            "ms_per_step": round(t_both * 1e3, 3),
            "overlap_frac": round(1.0 - max(0.0, t_both - t_c) / t_x, 4) if t_x > 0 else None,
            "hidden": bool(t_both <= 1.05 * max(t_c, t_x)),
            "h2d_gbs_wall": round(s3["h2d_bytes"] / dt / 1e9, 2),
            "frac_of_link_roofline": round(s3["h2d_bytes"] / dt / 1e9 / LINK_PEAK_GBS, 4),
            "d2h_bytes_per_step": int(s3["d2h_bytes"] / K), "host_wait_s": round(s3["host_wait_s"], 4),
            "host_enqueue_ms_per_step": round(s3["host_enqueue_s"] / K * 1e3, 4)}
    sweep = None
    if args.sweep:
        sweep = []
        for sg in [1.0] + [2.0 ** -k for k in range(1, 8)] + [0.0]:
            run.restart(sg)
            for _ in range(n):
                i = run.t % n
                run.step(hin[i], hout[i], stream)
            sync()
            st.reset_stats()
            Ks = 3 * n
            t0 = time.perf_counter()
            for _ in range(Ks):
                i = run.t % n
                run.step(hin[i], hout[i], stream)
            sync()
            dts = time.perf_counter() - t0
            ss = st.get_stats()
            sweep.append({"sigma": sg, "streamed_seqs_per_mb": run.n_stream[0], "ms_per_step": round(dts / Ks * 1e3, 3),
                          "tokens_per_s": round(ss["tokens"] / dts, 1),
                          "h2d_gb_per_step": round(ss["h2d_bytes"] / Ks / 1e9, 4),
                          "h2d_gbs_wall": round(ss["h2d_bytes"] / dts / 1e9, 2)})
            log("sweep:", json.dumps(sweep[-1]))
    out = {
        "metric": "stage decode tokens/sec with host-offloaded KV", "value": round(value, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype,
        "data": "synthetic" if not args.no_writeback else "synthetic (DIAGNOSTIC RUN WITHOUT KV WRITE-BACK: not a result)",
        "config": {"workload": f"{shape.name}: {shape.n_layers} layers, hidden {shape.hidden}, "
                               f"{shape.n_q_heads}Q/{shape.n_kv_heads}KV heads x {shape.head_dim}, ffn {shape.ffn}, "
                               f"{n} micro-batches x {shape.seqs_per_mb} seqs, prompts {shape.ctx_lo}-{shape.ctx_hi} tokens",
                   "sigma": args.sigma, "schedule": "cyclic (execute D_i, prefetch D_i+1, overwrite D_i-1)",
                   "inactive_kv": "pinned host memory", "page_tokens": 16,
                   "prefetch_issue": (f"transfer orchestrator, {args.orchestrated:g} MiB chunks, window 2"
                                      if args.orchestrated > 0 else "stage's own prefetch stream, whole runs")},
        "roofline": roofline, "legs": legs,
    }
    if sweep is not None:
        out["sigma_sweep"] = sweep
    if args.probe_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            pm.probe_copy(dst.data_ptr(), src.data_ptr(), src.numel(), stream.cuda_stream)
        torch.cuda.synchronize()
        del src, dst
    if xfer is not None:
        st.attach_xfer(None)
        xfer.destroy()
    if not args.no_cpu_baseline:
        st.destroy()
        del run
        out["cpu_baseline"] = cpu_baseline(shape, syn, {0: syn.ctx_lens(0)}, min(args.cpu_seqs, shape.seqs_per_mb),
                                           args.cpu_steps)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
