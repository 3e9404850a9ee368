"""Fits the decode-time model  alpha*b + beta*L + delta  (Sec. 3.3.1, Eq. 2) to step times measured
on this GPU and checks it the way the paper does (Sec. 4.3: actual / predicted over 100 consecutive
decode steps).  Run:  python -m paper_2605_02189_amd.fit_estimator [--config C2]

Prints one JSON object: the fitted parameters, the fit residuals, the accuracy on 100 consecutive
steps of a ragged batch that was not part of the fit, the measured prefetch bandwidth B and the
prefetch budget B * T_hat (Eq. 6) for the configuration's own micro-batch.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="C2")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--verbose", action="store_true")
    args = ap.parse_args()
    import torch
    from . import binding as pm, estimator as est
    from .harness import StageRunner
    from .synth_inputs import CONFIGS, SynthInputs

    base = CONFIGS[args.config]
    bs = [max(1, base.seqs_per_mb // 4), (5 * base.seqs_per_mb) // 8, base.seqs_per_mb]
    # profiling batches: ragged prompt-length mixes (requests of a real workload never share a length;
    # the attention kernel's load balance depends on it), three batch sizes x three length ranges
    Ls = [(256, 1024), (256, 4096), (1024, 4096)]
    grid = [(b, L) for b in bs for L in Ls]
    n = len(grid) + 1
    rng = np.random.default_rng(args.seed)
    ctx = {k: rng.integers(lo, hi + 1, size=b).astype(np.int32) for k, (b, (lo, hi)) in enumerate(grid)}
    ctx[n - 1] = rng.integers(512, 4097, size=base.seqs_per_mb).astype(np.int32)      # evaluation batch (not fitted)
    shape = base.with_(n_microbatches=n)
    syn = SynthInputs(shape, seed=args.seed)
    run = StageRunner(shape, syn, sigma=0.0, steps=120 * n, ctx_lens=ctx, gpu_pool_all_resident=True)
    st = run.stage
    run.load()
    stream = torch.cuda.Stream()        # a real stream handle: the default stream's handle is 0, which the
    sp = stream.cuda_stream             # library reads as "use your own compute stream"
    # prefetch bandwidth B: the largest micro-batch, timed on its own
    big = int(np.argmax([int(c.sum()) for c in ctx.values()]))
    st.sync()
    s0 = st.get_stats()
    t0 = time.perf_counter()
    st.prefetch_kv(big)
    st.sync()
    dt = time.perf_counter() - t0
    B = (st.get_stats()["h2d_bytes"] - s0["h2d_bytes"]) / dt
    for mb in range(n):
        st.prefetch_kv(mb)
    st.sync()
    hin = {mb: run.hidden_tensor(mb, mb) for mb in range(n)}
    hout = {mb: torch.empty_like(hin[mb]) for mb in range(n)}

    def timed_steps(mb, count):
        out = []
        for _ in range(count):
            L = int(st.get_ctx_lens(mb).sum())
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            st.decode_step(mb, hin[mb].data_ptr(), hout[mb].data_ptr(), sp)
            e1.record(stream)
            e1.synchronize()
            out.append((len(ctx[mb]), L, e0.elapsed_time(e1) * 1e-3))
        return out

    samples = []
    for mb in range(n - 1):
        timed_steps(mb, 3)
        samples += timed_steps(mb, 8)
    if args.verbose:
        for smp in samples:
            print("sample b=%d L=%d t=%.3f ms" % (smp[0], smp[1], smp[2] * 1e3), file=sys.stderr)
    b_, L_, t_ = (np.array(x) for x in zip(*samples))
    model = est.fit(b_, L_, t_)
    fit_acc = est.accuracy(model, b_, L_, t_)
    timed_steps(n - 1, 3)
    ev = timed_steps(n - 1, 100)
    eb, eL, et = (np.array(x) for x in zip(*ev))
    ev_acc = est.accuracy(model, eb, eL, et)
    own_L = base.seqs_per_mb * (base.ctx_lo + base.ctx_hi) // 2
    sched = model.scheduler(link_tokens_per_s=B / base.kv_bytes_per_token)     # Eq. 2 / Eq. 6 live in the scheduler
    t_hat = sched.predict(base.seqs_per_mb, own_L)
    budget_tokens = sched.budget(t_hat)
    sched.destroy()
    out = {
        "config": base.name, "grid_b": bs, "grid_prefix_len_ranges": Ls,
        "alpha_us_per_request": model.alpha * 1e6, "beta_ns_per_token": model.beta * 1e9, "delta_ms": model.delta * 1e3,
        "fit": fit_acc, "eval_100_consecutive_steps_ragged_batch": ev_acc,
        "eval_batch": {"b": int(eb[0]), "L_first": int(eL[0]), "L_last": int(eL[-1]),
                       "ms_first": float(et[0] * 1e3), "ms_last": float(et[-1] * 1e3)},
        "B_prefetch_gbs": B / 1e9,
        "own_microbatch": {"b": base.seqs_per_mb, "L": int(own_L), "t_hat_ms": t_hat * 1e3,
                           "budget_mb": budget_tokens * base.kv_bytes_per_token / 1e6,
                           "budget_tokens": budget_tokens,
                           "sigma_star": min(1.0, budget_tokens / max(own_L, 1))},
    }
    print(json.dumps(out))
    st.destroy()


if __name__ == "__main__":
    main()
