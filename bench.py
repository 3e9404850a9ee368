#!/usr/bin/env python3
"""Benchmark of the stage-decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config C5] [--sigma 1.0]
    python bench.py --probes          # HBM stream rate and host-link rates only (one JSON line of their own)

A step = one pass of the whole hot path over one micro-batch: pipemax_decode_step of D_i with the KV prefetch of
D_{i+1} and the write-back running beside it (cyclic schedule, Eq. 3).  The default workload is the largest
configuration, configs[4] (C5: 10 of 80 layers of a 70B-shaped model, 8 micro-batches x 256 sequences x 4096-token
contexts, bf16, 344 GB of KV: more than the HBM holds, so it is streamed from pinned host memory), with every
inactive micro-batch's KV in host memory (sigma = 1).  A process here can pin about 64 GiB, so only as many
micro-batches as fit get host pages and KV of their own; the others are aliases (pipemax_mb_define_alias: same
lengths, the same host pages, GPU pages of their own): the transfers move the same bytes along the same access
pattern and the kernels read the same amount of KV.  config.workload says how many are aliases.  Weights, hidden
states and the active micro-batch's pages (once prefetched) are resident in HBM when the timed region starts; the
KV of the inactive micro-batches is in host memory by construction: moving it is the method being measured.

Prints ONE JSON line.  Besides the headline (tokens/s of the streamed schedule) it carries
  roofline      achieved HBM GB/s of the attention kernel from the dispatches' own start / stop events,
  cpu_baseline  the CPU oracle timed on a bounded sample of the same workload,
  legs          compute-only / transfers-only / both, both overlap figures and the link rate,
  sigma_sweep   step time against the streamed fraction sigma of every micro-batch, with the crossover from
                link-bound to HBM-bound and whether the transfers are hidden there,
  also          (default run only) the same figures, compact, for configs[3] (C4).
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
PIN_BUDGET_GIB = 60.0          # pinned host memory the page pool may take (a process here pins about 64 GiB)


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


def cpu_baseline(shape, syn, ctx0, k_seqs, budget_s):
    """The oracle as it stands on a sample of micro-batch 0: k sequences, all layers, full context; as many decode
    steps as fit the time budget (at least one)."""
    from oracle.stage_oracle import StageOracle
    orc = StageOracle(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                      shape.ffn, shape.rope_base, shape.rms_eps)
    for l in range(shape.n_layers):
        orc.set_layer_weights(l, **{k: syn.as_f32(v) for k, v in syn.weights(l).items()})
    seqs = list(range(k_seqs))
    for s in seqs:
        kv = [syn.kv_prefix(0, s, l, int(ctx0[s])) for l in range(shape.n_layers)]
        orc.define_sequence(0, s, [syn.as_f32(k) for k, _ in kv], [syn.as_f32(v) for _, v in kv])
    x = syn.as_f32(syn.hidden(0, shape.seqs_per_mb))[seqs]
    orc.decode_step(0, x, seqs=seqs)                      # untimed first step (page-in, BLAS start-up)
    n_steps, t0 = 0, time.perf_counter()
    while True:
        orc.decode_step(0, x, seqs=seqs)
        n_steps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or n_steps >= 64:
            break
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
    return {"value": round(k_seqs * n_steps / dt, 2), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{n_steps} decode steps ({dt:.1f} s) of {k_seqs} of the {shape.seqs_per_mb} sequences of "
                      f"micro-batch 0, all {shape.n_layers} layers, full {int(ctx0[0])}-token context, fp32"}


def run_probes(args):
    """The rates the roofline arguments lean on, measured with the library's probe entry points."""
    import torch
    from paper_2605_02189_amd import binding as pm
    out = {"probe": "hbm stream + host link", "unit": "GB/s"}
    n = 4 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_()
    dst = torch.empty(n, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    sp = torch.cuda.current_stream().cuda_stream

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        best = 1e9
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            best = min(best, a.elapsed_time(b) * 1e-3)
        return best
    hbm = {}
    for name, seg in (("grid_stride", 0), ("contiguous_8KiB_per_group", 2), ("contiguous_64KiB_per_group", 16),
                      ("contiguous_1MiB_per_group", 256)):
        hbm["read_" + name] = round(n / timed(lambda: pm.probe_read(src.data_ptr(), n, seg, sink.data_ptr(), sp)) / 1e9, 1)
    hbm["copy_read_plus_write"] = round(2 * n / timed(lambda: pm.probe_copy(dst.data_ptr(), src.data_ptr(), n, sp)) / 1e9, 1)
    out["hbm_gbs"] = hbm
    log("hbm:", json.dumps(hbm))
    del src, dst
    torch.cuda.empty_cache()
    link = {}
    total = 2 << 30
    for name, direction in (("h2d", 0), ("d2h", 1), ("both", 2)):
        r = pm.probe_link(total, 64 << 20, None, direction, repeats=3)
        link[name + "_64MiB_pieces"] = {"h2d": round(r["h2d_bytes"] / r["h2d_s"] / 1e9, 2) if r["h2d_s"] else None,
                                        "d2h": round(r["d2h_bytes"] / r["d2h_s"] / 1e9, 2) if r["d2h_s"] else None}
    # block-first (whole pages and merged runs of pages) against layer-first fragments (Sec. 4.4): one hipMemcpyAsync
    # per piece, pieces one page apart for the fragments (the other layers of the page lie between them)
    pieces = {}
    for label, piece, stride in (("run_64MiB (block-first, merged page runs)", 64 << 20, None),
                                 ("page_640KiB (block-first, one copy per page, 70B stage)", 640 << 10, None),
                                 ("page_512KiB (block-first, one copy per page, 8B stage)", 512 << 10, None),
                                 ("fragment_64KiB (layer-first, K+V of one layer of a page)", 64 << 10, 640 << 10),
                                 ("fragment_32KiB (layer-first, K or V of one layer of a page)", 32 << 10, 320 << 10)):
        tot = min(total, piece * 16384)
        r = pm.probe_link(tot, piece, stride, 0, repeats=2)
        pieces[label] = round(r["h2d_bytes"] / r["h2d_s"] / 1e9, 2)
        log("link piece", label, pieces[label])
    # strided copies: one layer's 64 KiB block of each page of a run, out of block-first host pages (640 / 512 KiB
    # apart), into a packed device region -- the prefetch of a layer-major device pool
    for label, row, pitch, rows in (("2d_64KiB_rows_x257 (70B stage, one sequence of 4097 tokens, one layer)", 64 << 10, 640 << 10, 257),
                                    ("2d_64KiB_rows_x129 (70B stage, 2049 tokens)", 64 << 10, 640 << 10, 129),
                                    ("2d_64KiB_rows_x65 (8B stage, 1025 tokens)", 64 << 10, 512 << 10, 65),
                                    ("2d_64KiB_rows_x1024", 64 << 10, 640 << 10, 1024)):
        copies = max(1, min(2048, (2 << 30) // (row * rows)))
        r = pm.probe_link_2d(row, pitch, rows, copies, repeats=2)
        pieces[label] = round(r["h2d_bytes"] / r["h2d_s"] / 1e9, 2)
        log("link piece", label, pieces[label])
    link["h2d_by_piece"] = pieces
    out["link_gbs"] = link
    launch = {}
    for label, graph in (("one_by_one", False), ("captured_graph", True)):
        r = pm.probe_launch(41, graph, repeats=50)          # 41 = the launches of an 8-layer fused decode step
        launch[label] = {"host_enqueue_us_per_kernel": round(r["host_enqueue_s"] / 41 * 1e6, 2),
                         "gpu_us_per_kernel": round(r["gpu_s"] / 41 * 1e6, 2)}
    out["launch_chain_of_41_dependent_one_wave_kernels"] = launch
    log("launch:", json.dumps(launch))
    # Reference only, not part of the path: the vendor library's plain bf16 GEMM (torch.matmul) on the shapes of the
    # stage's four projections, four weight matrices taken in turn so that they stream from HBM; the time includes
    # the gap between launches, as a step's kernels do.
    lib = {}
    for label, rows, h, nqkv, f in (("8B-shaped stage, 64 rows", 64, 4096, 6144, 14336),
                                    ("70B-shaped stage, 256 rows", 256, 8192, 10240, 28672),
                                    ("70B-shaped stage, 1024 rows", 1024, 8192, 10240, 28672)):
        per = {}
        for gname, k, n_cols in (("qkv", h, nqkv), ("o", h, h), ("gate_up", h, 2 * f), ("down", f, h)):
            a = torch.randn(rows, k, device="cuda", dtype=torch.bfloat16)
            ws = [torch.randn(k, n_cols, device="cuda", dtype=torch.bfloat16) * 0.02 for _ in range(4)]
            reps = 40
            t = timed(lambda: [torch.matmul(a, ws[r % 4]) for r in range(reps)], reps=2) / reps
            per[gname] = {"us": round(t * 1e6, 1), "tflops": round(2 * rows * k * n_cols / t / 1e12, 1),
                          "weight_gbs": round(k * n_cols * 2 / t / 1e9, 1)}
            del a, ws
        per["layer_us"] = round(sum(v["us"] for v in per.values()), 1)
        lib[label] = per
        log("library gemm", label, json.dumps(per))
    out["library_gemm_reference"] = lib
    out["link_peak_nominal_gbs"] = LINK_PEAK_GBS
    out["hbm_peak_nominal_gbs"] = HBM_PEAK_GBS
    print(json.dumps(out), flush=True)


def run_config(name, args, *, light=False):
    """Sets one configuration up and measures it.  light: shorter timed run, no per-class breakdown."""
    import numpy as np
    import torch
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.harness import StageRunner, pages_for
    from paper_2605_02189_amd.synth_inputs import CONFIGS, SynthInputs

    shape = CONFIGS[name]
    if args.microbatches:
        shape = shape.with_(n_microbatches=args.microbatches)
    n, b = shape.n_microbatches, shape.seqs_per_mb
    K = args.steps if args.steps is not None else (2 * n if light else shape.decode_steps)
    W = args.warmup if args.warmup is not None else n
    sweep_sigmas = [] if args.no_sweep else [0.5, 0.25, 0.125, 1 / 16, 1 / 32, 1 / 64, 1 / 128, 0.0]
    Kc = min(K, 4 * n) if light else min(K, 8 * n)
    # cycles per sweep point: at least two, at most 24, about 0.15 s (guessing the step at 5 TB/s of HBM traffic)
    kv_guess = b * (shape.ctx_lo + shape.ctx_hi) // 2 * shape.kv_bytes_per_token
    sweep_cycles = max(2, min(24, int(0.15 / ((shape.weight_bytes + kv_guess) / 5e12) / n + 0.5)))
    total_steps = ((W + K) + (0 if args.no_legs else 2 * n + 3 * Kc + 2 * n)
                   + (len(sweep_sigmas) + 1) * (3 + sweep_cycles) * n + 2 * n)

    t_setup = time.perf_counter()
    syn = SynthInputs(shape, seed=args.seed)
    lens = {mb: syn.ctx_lens(mb) for mb in range(n)}
    steps_per_mb = -(-total_steps // n)
    grow = pages_for(steps_per_mb) + 1
    mb_bytes = [sum(pages_for(int(l)) + grow for l in lens[mb]) * shape.page_bytes for mb in range(n)]
    real = 0
    while real < n and sum(mb_bytes[: real + 1]) <= PIN_BUDGET_GIB * 2 ** 30:
        real += 1
    real = max(1, real)
    # GPU pool: every micro-batch resident if the HBM has room for them beside the weights, else as many as fit
    free_b, _ = torch.cuda.mem_get_info()
    room = free_b - shape.weight_bytes - (10 << 30)
    n_res = n
    while n_res > 2 and sum(sorted(mb_bytes, reverse=True)[:n_res]) > room:
        n_res -= 1
    run = StageRunner(shape, syn, sigma=args.sigma, steps=total_steps, real_microbatches=real,
                      gpu_resident_microbatches=n_res, arenas=args.arenas,
                      flags=(pm.FLAG_NO_WRITEBACK if args.no_writeback else 0)
                      | (pm.FLAG_DEVICE_LAYER_MAJOR if args.device_layout == "layer" else 0))
    st = run.stage
    xfer = None
    if args.orchestrated:      # the prefetch goes through the transfer orchestrator in chunks of that many MiB
        xfer = pm.Xfer(device=0, max_inflight_bulk=2, chunk_bytes=int(args.orchestrated) << 20)
        st.attach_xfer(xfer)
    run.load()
    hin = [run.hidden_tensor(mb, mb) for mb in range(n)]
    hout = [torch.empty_like(h) for h in hin]
    stream = torch.cuda.current_stream()
    kv_mb = sum(int(l) for l in run.ctx0[0]) * shape.kv_bytes_per_token
    log(f"setup {time.perf_counter() - t_setup:.1f}s: {name} engine={st.get_stats()['engine']} weights "
        f"{shape.weight_bytes / 1e9:.2f} GB, KV/mb {kv_mb / 1e9:.2f} GB, {real} of {n} micro-batches with host pages of "
        f"their own, GPU pool for {n_res} whole micro-batches")

    def sync():
        torch.cuda.synchronize()
        st.sync()

    def timed_steps(k):
        sync()
        st.reset_stats()
        t0 = time.perf_counter()
        for _ in range(k):
            i = run.t % n
            run.step(hin[i], hout[i], stream)
        sync()
        dt = time.perf_counter() - t0
        return dt, st.get_stats()

    res = {"name": name, "shape": shape, "n": n, "b": b, "K": K, "W": W, "real": real, "n_res": n_res}
    # ---- the timed run: compute + transfers, the literal configuration (sigma = 1 unless --sigma) --------------
    run.warm_start()
    for _ in range(W):
        i = run.t % n
        run.step(hin[i], hout[i], stream)
    dt, s3 = timed_steps(K)
    res.update(value=s3["tokens"] / dt, ms_per_step=dt / K * 1e3, dt=dt, s_both=s3)
    log(f"{name} sigma={args.sigma}: {dt / K * 1e3:.3f} ms/step, {s3['tokens'] / dt:.1f} tokens/s, "
        f"h2d {s3['h2d_bytes'] / dt / 1e9:.2f} GB/s")
    legs, roofline = {}, None
    if not args.no_legs:
        # ---- transfers only: the same evict / prefetch traffic, no kernels ---------------------------------
        sync()
        st.set_flags(pm.FLAG_TIME_KERNELS, 0)
        st.reset_stats()
        Kx = n if light else 2 * n
        t0 = time.perf_counter()
        for _ in range(Kx):
            run.step(None, None, stream, compute=False)
        sync()
        t_x = (time.perf_counter() - t0) / Kx
        s2 = st.get_stats()
        st.set_flags(0, pm.FLAG_TIME_KERNELS)
        link_gbs = s2["h2d_bytes"] / Kx / t_x / 1e9
        legs["transfer_only"] = {
            "ms_per_step": round(t_x * 1e3, 3), "h2d_bytes_per_step": int(s2["h2d_bytes"] / Kx),
            "h2d_copies_per_step": s2["h2d_copies"] / Kx,
            "h2d_gbs_busy": round(s2["h2d_bytes"] / max(s2["h2d_ms"], 1e-9) / 1e6, 2), "h2d_gbs_wall": round(link_gbs, 2)}
        log("transfer-only:", json.dumps(legs["transfer_only"]))
        # ---- compute only: n_res micro-batches resident, no transfers ----------------------------------------
        for mb in range(n):
            st.evict_kv(mb)
        sync()
        res_mbs = list(range(n_res))
        for mb in res_mbs:
            st.prefetch_kv(mb)
        sync()
        sp = stream.cuda_stream

        def compute_steps(k, count_bytes=False):
            nbytes = 0
            for q in range(k):
                i = res_mbs[q % n_res]
                if count_bytes:
                    nbytes += shape.n_layers * attn_bytes(shape, st.get_ctx_lens(i))
                st.decode_step(i, hin[i].data_ptr(), hout[i].data_ptr(), sp)
            return nbytes
        compute_steps(n_res)
        sync()
        # (a) only the attention kernel timed, by the dispatches' own start / stop events: the roofline figure
        st.set_flags(pm.FLAG_TIME_KERNELS | pm.FLAG_TIME_ATTN_ONLY, 0)
        st.reset_stats()
        bytes_attn = compute_steps(Kc, count_bytes=True)
        sync()
        s0 = st.get_stats()
        attn_launches = int(s0["kernel_launches"]["attn"])
        attn_ms = s0["kernel_ms"]["attn"] / max(attn_launches, 1)
        # (b) every kernel class bracketed: the per-class breakdown (the brackets themselves cost time)
        st.set_flags(pm.FLAG_TIME_KERNELS, pm.FLAG_TIME_ATTN_ONLY)
        st.reset_stats()
        t0 = time.perf_counter()
        compute_steps(Kc)
        sync()
        t_timed = time.perf_counter() - t0
        s1 = st.get_stats()
        st.set_flags(0, pm.FLAG_TIME_KERNELS)
        # (c) the same steps without any bracket: the compute-only step time
        sync()
        st.reset_stats()
        t0 = time.perf_counter()
        compute_steps(Kc)
        sync()
        t_c = (time.perf_counter() - t0) / Kc
        s_plain = st.get_stats()
        kms, kl = s1["kernel_ms"], s1["kernel_launches"]
        achieved = bytes_attn / max(attn_launches, 1) / (attn_ms * 1e-3) / 1e9
        lens_now = st.get_ctx_lens(0)
        _cp, _nch, per_wave = pm.plan_attention_chunks(
            b, shape.n_kv_heads, int(lens_now.max()) + 1, int(((lens_now + 1 + 15) // 16).sum()),
            torch.cuda.get_device_properties(0).multi_processor_count)
        roofline = {"bound": "hbm",
                    "kernel": ("k_attention (shape-generic paged decode attention, one work-group per query head)"
                               if st.get_stats()["engine"] == 0 else
                               "k_attn_w (GQA paged decode attention, a wave per (chunk, KV head, sequence) item)" if per_wave
                               else "k_attn (GQA paged decode attention, a work-group per (chunk, KV head, sequence) item)"),
                    "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic(name),
                    "traffic_measured_on_algorithmic_bytes": measured_traffic(name, "algorithmic_bytes_per_launch"),
                    "avg_launch_us": round(attn_ms * 1e3, 2), "launches": attn_launches,
                    "bytes_per_launch": int(bytes_attn / max(attn_launches, 1))}
        hbm_bytes_step = shape.weight_bytes + bytes_attn / Kc
        gemm_ms = (kms["gemm_qkv"] + kms["gemm_o"] + kms["gemm_gu"] + kms["gemm_d"]) / Kc
        legs["compute_only"] = {
            "ms_per_step": round(t_c * 1e3, 4), "tokens_per_s": round(b / t_c, 1),
            "resident_microbatches": n_res,
            "ms_per_step_with_event_brackets": round(t_timed / Kc * 1e3, 4),
            "hbm_bytes_per_step": int(hbm_bytes_step),
            "frac_of_hbm_roofline": round(hbm_bytes_step / t_c / 1e9 / HBM_PEAK_GBS, 4),
            # attention: the dispatch's own start and stop; the other classes: between two stream events, which
            # includes the gap to the next launch (about 3 us); exact durations: profiles/bench_<config>_kernel_trace.txt
            "kernel_us_per_launch": {k: round(kms[k] / max(kl[k], 1) * 1e3, 2) for k in kms if kl[k]},
            "kernel_ms_per_step": {k: round(kms[k] / Kc, 4) for k in kms if kl[k]},
            "gemm_tflops": round(2 * (shape.weight_bytes / shape.elem_bytes) * b / (gemm_ms * 1e-3) / 1e12, 1),
            "gemm_weight_gbs": round(shape.weight_bytes / (gemm_ms * 1e-3) / 1e9, 1),
            "host_enqueue_ms_per_step_with_event_brackets": round(s1["host_enqueue_s"] / Kc * 1e3, 4),
            "host_enqueue_ms_per_step": round(s_plain["host_enqueue_s"] / Kc * 1e3, 4)}
        log("compute-only:", json.dumps(legs["compute_only"]))
        t_both = dt / K
        legs["both"] = {
            "ms_per_step": round(t_both * 1e3, 3),
            # the survey's figure (written for the compute-bound regime) and a symmetric one: the share of the
            # shorter of the two activities that runs under the longer one
            "overlap_frac": round(1.0 - max(0.0, t_both - t_c) / t_x, 4) if t_x > 0 else None,
            "overlap_frac_symmetric": round(1.0 - max(0.0, t_both - max(t_c, t_x)) / min(t_c, t_x), 4),
            "hidden": bool(t_both <= 1.05 * max(t_c, t_x)),
            "h2d_gbs_wall": round(s3["h2d_bytes"] / dt / 1e9, 2),
            "frac_of_link_roofline": round(s3["h2d_bytes"] / dt / 1e9 / LINK_PEAK_GBS, 4),
            "frac_of_measured_link": round(s3["h2d_bytes"] / dt / 1e9 / link_gbs, 4),
            "d2h_bytes_per_step": int(s3["d2h_bytes"] / K), "host_wait_s": round(s3["host_wait_s"], 4),
            "host_enqueue_ms_per_step": round(s3["host_enqueue_s"] / K * 1e3, 4)}
        res.update(t_c=t_c, t_x=t_x, link_gbs=link_gbs)
    sweep = None
    if sweep_sigmas and not args.no_legs:
        # ---- step time against the streamed fraction; sigma shrinks, so only the newly resident part moves ----
        t_c, link_gbs = res["t_c"], res["link_gbs"]
        pool_pages = st.get_stats()["gpu_pages_total"]
        per_seq = pages_for(int(max(int(c.max()) for c in run.ctx0.values()))) + grow
        sweep = [{"sigma": args.sigma, "ms_per_step": round(res["ms_per_step"], 3),
                  "h2d_gb_per_step": round(s3["h2d_bytes"] / K / 1e9, 4), "feasible": True}]
        full = {mb: [pages_for(int(l)) + grow for l in run.ctx0[mb]] for mb in range(n)}

        def pages_needed(ns):
            return (sum(sum(full[mb][: b - ns]) for mb in range(n))
                    + sum(sorted((sum(full[mb][b - ns:]) for mb in range(n)), reverse=True)[: run.arenas]) + 8)
        # where the HBM cannot hold every point of the list, the smallest streamed fraction it can hold joins it
        if pages_needed(0) > pool_pages:
            ns_min = next(k for k in range(b + 1) if pages_needed(k) <= pool_pages)
            sg_min = ns_min / b
            if ns_min < b and all(abs(sg_min - x) > 1e-9 for x in sweep_sigmas):
                sweep_sigmas = sorted(sweep_sigmas + [sg_min], reverse=True)
        for sg in sweep_sigmas:
            ns = int(round(sg * b))
            need = pages_needed(ns)
            if need > pool_pages:
                sweep.append({"sigma": sg, "feasible": False,
                              "why": f"resident parts + two streamed arenas need {need} GPU pages, the HBM holds {pool_pages}"})
                continue
            run.restart(sg)
            for _ in range(n):
                i = run.t % n
                run.step(hin[i], hout[i], stream)
            # at least two cycles and at least ~0.15 s, so that the drain at the end does not weigh on short steps
            est = max(t_c, ns * per_seq * shape.page_bytes / (link_gbs * 1e9))
            ks = n * max(2, min(sweep_cycles, int(0.15 / est / n + 0.5)))
            dts, ss = timed_steps(ks)
            row = {"sigma": sg, "feasible": True, "streamed_seqs_per_mb": ns, "steps": ks,
                   "ms_per_step": round(dts / ks * 1e3, 3),
                   "h2d_gb_per_step": round(ss["h2d_bytes"] / ks / 1e9, 4),
                   "host_wait_s": round(ss["host_wait_s"], 4)}
            # one more cycle with the attention launches and the wait for the prefetch timed (dispatch stamps and
            # events on the compute stream): where a step that is longer than the compute-only one loses its time
            st.set_flags(pm.FLAG_TIME_KERNELS | pm.FLAG_TIME_ATTN_ONLY, 0)
            _, sd = timed_steps(2 * n)
            st.set_flags(0, pm.FLAG_TIME_KERNELS | pm.FLAG_TIME_ATTN_ONLY)
            row["attn_us_per_launch"] = round(sd["kernel_ms"]["attn"] / max(sd["kernel_launches"]["attn"], 1) * 1e3, 2)
            row["prefetch_stall_ms_per_step"] = round(sd["prefetch_stall_ms"] / (2 * n), 4)
            sweep.append(row)
            log("sweep:", json.dumps(sweep[-1]))
        # the compute-only reference of the sweep is its own sigma = 0 point (same driver loop, same timing) where
        # the pool can hold it, else the compute-only leg
        zero = [p for p in sweep if p["feasible"] and p["sigma"] == 0.0]
        t_ref = zero[0]["ms_per_step"] * 1e-3 if zero else t_c
        for p in sweep:
            if not p["feasible"]:
                continue
            tx = p["h2d_gb_per_step"] / link_gbs        # what the step's prefetch takes on the link alone (s)
            p["t_transfer_ms_at_measured_link"] = round(tx * 1e3, 3)
            p["bound"] = "link" if tx > t_ref else "hbm"
            p["hidden"] = bool(p["ms_per_step"] * 1e-3 <= 1.05 * max(t_ref, tx))
            p["vs_compute_only"] = round(p["ms_per_step"] * 1e-3 / t_ref, 3)
        sigma_star = t_ref * link_gbs * 1e9 / kv_mb
        hbm_side = [p for p in sweep if p["feasible"] and p["bound"] == "hbm" and p["sigma"] > 0]
        link_side = [p for p in sweep if p["feasible"] and p["bound"] == "link"]
        res["crossover"] = {
            "sigma_star_predicted": round(sigma_star, 4),
            "formula": "sigma* = T_compute_only * link rate / KV bytes of one micro-batch",
            "t_compute_only_ms_used": round(t_ref * 1e3, 4),
            "smallest_link_bound_sigma_measured": min((p["sigma"] for p in link_side), default=None),
            "largest_hbm_bound_sigma_measured": max((p["sigma"] for p in hbm_side), default=None),
            "hidden_at_largest_hbm_bound_sigma": (max(hbm_side, key=lambda p: p["sigma"])["hidden"] if hbm_side else None),
            "reachable": bool(hbm_side),
        }
    res.update(legs=legs, roofline=roofline, sweep=sweep, syn=syn, ctx0=run.ctx0[0])
    if xfer is not None:
        st.attach_xfer(None)
        xfer.destroy()
    st.destroy()
    del run
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", default=None, help="C1..C5 (default: C5, with a compact C4 run beside it)")
    ap.add_argument("--sigma", type=float, default=1.0, help="streamed fraction of every micro-batch")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--microbatches", type=int, default=None,
                    help="run with fewer micro-batches than the configuration names")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-legs", action="store_true", help="skip the compute-only / transfer-only legs and the sweep")
    ap.add_argument("--no-sweep", action="store_true", help="skip the sweep over the streamed fraction")
    ap.add_argument("--no-also", action="store_true", help="default run: skip the compact C4 run")
    ap.add_argument("--no-writeback", action="store_true", help="diagnostic: skip the KV write-back (invalid as a result)")
    ap.add_argument("--orchestrated", type=int, default=0, metavar="MiB",
                    help="route the KV prefetch through the transfer orchestrator in chunks of this many MiB (block-first pool only)")
    ap.add_argument("--arenas", type=int, default=2,
                    help="GPU room for this many streamed parts: 2 = Eq. 3 (the prefetch overwrites D_i-1), 3 = it "
                         "overwrites D_i-2 and never waits for the compute stream")
    ap.add_argument("--device-layout", choices=["block", "layer"], default="block",
                    help="GPU page pool block-first (as the host replica) or [layer][page]")
    ap.add_argument("--probes", action="store_true", help="only the HBM stream / host link probes")
    ap.add_argument("--probe-copy", action="store_true",
                    help="also launch the library's plain copy kernel (256 MiB, 3 times): calibration for --pmc runs")
    ap.add_argument("--cpu-seqs", type=int, default=8)
    ap.add_argument("--cpu-budget-s", type=float, default=15.0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one pipeline stage on ONE GPU; --gpus must be 1 "
              "(the stages of a pipeline are independent processes, one per GPU; nothing here runs on a second GPU)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_02189_amd.build import ensure_built
    ensure_built()      # loads what is built; builds only if nothing is
    from paper_2605_02189_amd import binding as pm
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    if args.probes:
        run_probes(args)
        return

    name = args.config or "C5"
    r = run_config(name, args)
    shape, n = r["shape"], r["n"]
    out = {
        "metric": "stage decode tokens/sec with host-offloaded KV", "value": round(r["value"], 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": r["K"], "warmup": r["W"], "ms_per_step": round(r["ms_per_step"], 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype,
        "data": "synthetic" if not args.no_writeback else "synthetic (DIAGNOSTIC RUN WITHOUT KV WRITE-BACK: not a result)",
        "config": {"workload": f"{shape.name}: {shape.n_layers} layers, hidden {shape.hidden}, "
                               f"{shape.n_q_heads}Q/{shape.n_kv_heads}KV heads x {shape.head_dim}, ffn {shape.ffn}, "
                               f"{n} micro-batches x {shape.seqs_per_mb} seqs, prompts {shape.ctx_lo}-{shape.ctx_hi} tokens; "
                               f"{r['real']} micro-batches with pinned host pages of their own, {n - r['real']} aliases "
                               f"of them (same lengths and host pages, own GPU pages)",
                   "sigma": args.sigma, "schedule": "cyclic (execute D_i, overwrite D_i-1, prefetch D_i+1)",
                   "inactive_kv": "pinned host memory", "page_tokens": 16, "gpu_arenas_for_streamed_kv": args.arenas,
                   "gpu_pool_layout": "[layer][page]" if args.device_layout == "layer" else "block-first pages",
                   "prefetch_issue": (f"transfer orchestrator, chunks of {args.orchestrated} MiB, two in flight"
                                      if args.orchestrated else
                                      "stage's prefetch worker, whole page runs on the prefetch stream")},
        "roofline": r["roofline"], "legs": r["legs"],
    }
    if r["sweep"] is not None:
        out["sigma_sweep"] = r["sweep"]
        out["crossover"] = r["crossover"]
    if args.config is None and not args.no_also:
        import copy
        a2 = copy.copy(args)
        a2.steps, a2.warmup = None, None
        c4 = run_config("C4", a2, light=True)
        out["also"] = {"C4": {
            "workload": f"C4: 10 layers, 8 micro-batches x 256 seqs x 2048-token prompts; {c4['real']} with host pages of "
                        f"their own, {c4['n'] - c4['real']} aliases",
            "tokens_per_s": round(c4["value"], 1), "ms_per_step": round(c4["ms_per_step"], 3), "steps": c4["K"],
            "sigma": args.sigma, "roofline": c4["roofline"],
            "compute_only_ms_per_step": c4["legs"].get("compute_only", {}).get("ms_per_step"),
            "compute_only_tokens_per_s": c4["legs"].get("compute_only", {}).get("tokens_per_s"),
            "frac_of_hbm_roofline": c4["legs"].get("compute_only", {}).get("frac_of_hbm_roofline"),
            "both": c4["legs"].get("both"),
            "sigma_sweep": [{k: p.get(k) for k in ("sigma", "ms_per_step", "bound", "hidden", "vs_compute_only", "feasible")}
                            for p in (c4["sweep"] or [])],
            "crossover": c4.get("crossover")}}
    if args.probe_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            pm.probe_copy(dst.data_ptr(), src.data_ptr(), src.numel(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, r["syn"], r["ctx0"], min(args.cpu_seqs, shape.seqs_per_mb),
                                           args.cpu_budget_s)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
