"""The decode-time estimator on the GPU (Sec. 3.3.1, Eq. 2; the bar of Sec. 4.3: actual / predicted over 100
consecutive decode steps, more than 90 % of them within 5 % and the worst below 8 %) and the prefetch budget it
feeds (Sec. 3.3.2, Eq. 6), on the 8B-shaped stage (8 layers: with fewer the time of a step that is enqueued and
awaited on its own is the host's launch time, not the GPU's): the model is fitted by least squares on step
times of six ragged profiling batches (two batch sizes x three length ranges) and then checked on 100 consecutive
steps of a ragged batch that was not part of the fit, during which its total length grows by 6400 tokens."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_fitted_model_predicts_100_consecutive_steps_of_an_unseen_batch():
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    from oracle import scheduler_oracle as so
    from paper_2605_02189_amd import estimator as est
    from paper_2605_02189_amd.harness import StageRunner
    from paper_2605_02189_amd.synth_inputs import CONFIGS, SynthInputs

    base = CONFIGS["C2"]
    grid = [(b, L) for b in (16, 64) for L in ((256, 1024), (256, 4096), (1024, 4096))]
    n = len(grid) + 1
    rng = np.random.default_rng(0)
    ctx = {k: rng.integers(lo, hi + 1, size=b).astype(np.int32) for k, (b, (lo, hi)) in enumerate(grid)}
    ctx[n - 1] = rng.integers(512, 4097, size=base.seqs_per_mb).astype(np.int32)      # evaluation batch (not fitted)
    shape = base.with_(n_microbatches=n)
    syn = SynthInputs(shape, seed=0)
    run = StageRunner(shape, syn, sigma=0.0, steps=120 * n, ctx_lens=ctx, gpu_pool_all_resident=True)
    st = run.stage
    run.load()
    assert st.get_stats()["engine"] == 1
    stream = torch.cuda.Stream()
    sp = stream.cuda_stream
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
    b_, L_, t_ = (np.array(x) for x in zip(*samples))
    model = est.fit(b_, L_, t_)
    print(f"alpha {model.alpha * 1e6:.2f} us/request, beta {model.beta * 1e9:.2f} ns/token, delta {model.delta * 1e3:.3f} ms",
          flush=True)
    assert model.beta > 0 and model.delta > 0          # attention time grows with the context; a step has a fixed part
    timed_steps(n - 1, 3)
    ev = timed_steps(n - 1, 100)
    eb, eL, et = (np.array(x) for x in zip(*ev))
    acc = est.accuracy(model, eb, eL, et)
    print("100 consecutive steps of the unseen batch:", acc, f"L {eL[0]} -> {eL[-1]}", flush=True)
    assert eL[-1] - eL[0] == 99 * base.seqs_per_mb
    assert acc["within_5pct"] >= 0.90, acc
    assert acc["worst_dev"] < 0.08, acc
    # the budget this model gives the scheduler (Eq. 6): the C ABI's evaluation against the oracle's formulas
    link_tokens_per_s = 56.0e9 / base.kv_bytes_per_token
    sched = model.scheduler(link_tokens_per_s=link_tokens_per_s, n_batches=4)
    for b, L in ((int(eb[0]), int(eL[0])), (int(eb[-1]), int(eL[-1])), (16, 9000)):
        t_hat = sched.predict(b, L)
        assert t_hat == so.predict_time(model.alpha, model.beta, model.delta, b, L)
        assert sched.budget(t_hat) == so.budget_tokens(link_tokens_per_s, t_hat)
        assert 0 < sched.budget(t_hat) < L + 10**6
    sched.destroy()
    st.destroy()
