"""Prefetch-aware scheduler against static prefetching on this GPU (the comparison of Sec. 4.3, Fig. 9):
the same stage, the same requests and the same selection code; only the prefetch budget differs --
B * T_hat of the executing batch (Eq. 6) for the scheduler, a fixed fraction of the GPU KV pool for the
static policies.  Run:  python -m paper_2605_02189_amd.sched_experiment [--mix sharegpt|longbench]

Requests: n batches x 64 requests whose prefix lengths follow the shape of the paper's Table 2 (lognormal
input and output lengths with the table's mean and median for the ShareGPT-like mix; a symmetric input
length around the table's mean plus a lognormal output for the LongBench-like mix); no dataset item is used.
The GPU KV pool holds a fraction of all cached tokens (--pool-frac), the rest lives in pinned host memory.
Prints one JSON object: per policy the tokens/s over --iters iterations of Alg. 1, mean batch size, mean
prefetched tokens and the time per iteration.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np


def lognormal(rng, mean, median, size):
    sigma = np.sqrt(2.0 * np.log(mean / median))
    return rng.lognormal(np.log(median), sigma, size)


def prefix_lengths(mix: str, n: int, rng) -> np.ndarray:
    """Prefix length of a request caught at a uniformly random point of its decode phase."""
    if mix == "sharegpt":
        l_in, l_out = lognormal(rng, 343.76, 148.0, n), lognormal(rng, 237.20, 152.0, n)
        hi = 4096
    else:
        l_in, l_out = rng.normal(2686.89, 700.0, n), lognormal(rng, 101.78, 19.0, n)
        hi = 6144
    L = l_in + rng.random(n) * l_out
    return np.clip(np.rint(L), 16, hi).astype(np.int32)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="C2")
    ap.add_argument("--mix", default="sharegpt", choices=["sharegpt", "longbench"])
    ap.add_argument("--iters", type=int, default=240, help="timed iterations of Alg. 1 per policy")
    ap.add_argument("--warmup-iters", type=int, default=40,
                    help="untimed iterations before them (code loading, first touches, the scheduler's warm-up phase)")
    ap.add_argument("--pool-frac", type=float, default=0.75)
    ap.add_argument("--seed", type=int, default=0)
    # Eq. 2 parameters and B as fitted / measured by fit_estimator on this GPU for the C2 stage
    ap.add_argument("--alpha-us", type=float, default=2.7)
    ap.add_argument("--beta-ns", type=float, default=6.3)
    ap.add_argument("--delta-ms", type=float, default=0.87)
    ap.add_argument("--link-gbs", type=float, default=0.0,
                    help="effective host-to-device bandwidth B of Eq. 6; 0 = measure it first on this workload's own "
                         "prefetch copies (bytes / busy time of the copies of a calibration run)")
    ap.add_argument("--static", default="0.005,0.01,0.025,0.05,0.10,0.15,0.20,0.25")
    ap.add_argument("--verbose", action="store_true")
    args = ap.parse_args()
    import torch
    from . import binding as pm
    from .harness import StageRunner, pages_for
    from .synth_inputs import CONFIGS, SynthInputs

    base = CONFIGS[args.config]
    n, b = base.n_microbatches, base.seqs_per_mb
    rng = np.random.default_rng(args.seed)
    L = prefix_lengths(args.mix, n * b, rng)
    part = np.array(pm.sched_partition(L, n))                    # initial partition of Sec. 3.3.2
    ctx = {k: L[part == k] for k in range(n)}
    all_iters = args.iters + args.warmup_iters
    per_mb_steps = -(-all_iters // n)
    total_pages = int(sum(pages_for(l + per_mb_steps) for l in L))
    pool_pages = int(args.pool_frac * total_pages)
    shape = base.with_(n_microbatches=n)
    syn = SynthInputs(shape, seed=args.seed)
    stream = torch.cuda.Stream()
    kv_tok = base.kv_bytes_per_token
    model = dict(alpha_s=args.alpha_us * 1e-6, beta_s=args.beta_ns * 1e-9, delta_s=args.delta_ms * 1e-3,
                 link_tokens_per_s=(args.link_gbs or 56.0) * 1e9 / kv_tok, n_batches=n)

    def run_policy(static_tokens: int, time_copies: bool = False) -> dict:
        # a fresh stage per policy: every policy sees the same requests at the same lengths
        run = StageRunner(shape, syn, sigma=0.0, steps=all_iters, ctx_lens=ctx, gpu_pages=pool_pages,
                          flags=(pm.FLAG_TIME_KERNELS | pm.FLAG_TIME_ATTN_ONLY) if time_copies else 0)
        st = run.stage
        run.load()
        hin = run.hidden_tensor(0, 0)
        hout = torch.empty_like(hin)
        # every batch gets an equal share of the pool, filled in request order, less some headroom for the
        # first steps' new pages
        share = pool_pages // n - b // 4
        for k in range(n):
            used, ids = 0, []
            for s_, l in enumerate(ctx[k]):
                p = pages_for(int(l))
                if used + p > share:
                    break
                used += p
                ids.append(s_)
            st.prefetch_kv(k, ids)
        st.sync()
        sched = pm.Scheduler(static_budget_tokens=static_tokens, **model)
        sched.attach(st)
        tok = pf = bud = steady = npf = nev = 0
        bsz = []
        t0 = 0.0
        for t in range(all_iters):
            if t == args.warmup_iters:
                st.sync()
                st.reset_stats()
                lens0 = np.concatenate([st.get_ctx_lens(k) for k in range(n)])
                t0 = time.perf_counter()
            d = sched.iterate(st, t, hin.data_ptr(), hout.data_ptr(), stream.cuda_stream)
            if t < args.warmup_iters:
                continue
            tok += d["n_exec"]
            pf += d["prefetch_tokens"]
            bud += d["budget_tokens"]
            steady += d["steady"]
            npf += d["n_prefetch"]
            nev += d["n_evict"]
            bsz.append(d["n_exec"])
        st.sync()
        dt = time.perf_counter() - t0
        stats = st.get_stats()
        # tokens every request decoded in the timed iterations: a request that stays on the host never executes
        progress = np.concatenate([st.get_ctx_lens(k) for k in range(n)]) - lens0
        sched.destroy()
        st.destroy()
        return {"tokens_per_s": tok / dt, "ms_per_iter": dt / args.iters * 1e3, "mean_batch": float(np.mean(bsz)),
                "min_batch": int(min(bsz)), "requests_never_executed": int((progress == 0).sum()),
                "min_tokens_per_request": int(progress.min()), "median_tokens_per_request": float(np.median(progress)),
                "prefetch_tokens_per_iter": pf / args.iters,
                "budget_tokens_per_iter": bud / args.iters, "steady_frac": steady / args.iters,
                "h2d_gb_per_iter": stats["h2d_bytes"] / args.iters / 1e9,
                "h2d_copies_per_iter": stats["h2d_copies"] / args.iters,
                "requests_prefetched_per_iter": npf / args.iters, "requests_released_per_iter": nev / args.iters,
                "h2d_busy_ms_per_iter": stats["h2d_ms"] / args.iters,
                "prefetch_stall_ms_per_iter": stats["prefetch_stall_ms"] / args.iters,
                "host_wait_ms_per_iter": stats["host_wait_s"] / args.iters * 1e3,
                "host_enqueue_ms_per_iter": stats["host_enqueue_s"] / args.iters * 1e3}

    out = {"config": base.name, "mix": args.mix, "requests": int(n * b), "mean_prefix": float(L.mean()),
           "median_prefix": float(np.median(L)), "total_tokens": int(L.sum()), "pool_frac": args.pool_frac,
           "pool_tokens": pool_pages * 16, "iters": args.iters, "warmup_iters": args.warmup_iters, "model": model, "policies": {}}
    # The first stage of a process runs about 0.2 ms per iteration slower, so the first run is not a result; it
    # serves as the calibration of B: the prefetch copies of this workload are per request, a few MB each and
    # scattered over the GPU pool, and the rate they reach -- bytes over the time the copies of an iteration take
    # from the first one's start to the last one's end -- is what Eq. 6 calls the effective bandwidth.
    cal = run_policy(int(0.02 * pool_pages * 16), time_copies=True)
    b_eff = cal["h2d_gb_per_iter"] / max(cal["h2d_busy_ms_per_iter"], 1e-9) * 1e3
    out["calibration"] = {"static_budget_frac": 0.02, "h2d_gb_per_iter": cal["h2d_gb_per_iter"],
                          "h2d_busy_ms_per_iter": cal["h2d_busy_ms_per_iter"], "effective_link_gbs": b_eff,
                          "ms_per_iter": cal["ms_per_iter"],
                          "prefetch_stall_ms_per_iter": cal["prefetch_stall_ms_per_iter"]}
    if not args.link_gbs:
        model["link_tokens_per_s"] = b_eff * 1e9 / kv_tok
    out["model"] = model
    res = run_policy(0)
    out["policies"]["scheduler"] = res
    if args.verbose:
        print("scheduler", res, file=sys.stderr, flush=True)
    for f in [float(x) for x in args.static.split(",") if x]:
        res = run_policy(int(f * pool_pages * 16))
        out["policies"][f"static_{f:g}"] = res
        if args.verbose:
            print(f"static {f:g}", res, file=sys.stderr, flush=True)
    statics = [v["tokens_per_s"] for k, v in out["policies"].items() if k != "scheduler"]
    if statics:
        out["scheduler_vs_best_static"] = out["policies"]["scheduler"]["tokens_per_s"] / max(statics)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
