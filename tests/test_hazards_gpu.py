"""Stream / event hazards of the three-stream executor, forced from the host: injected delays on the
side streams and in the re-layout worker must not change any result, and pages that no live sequence
owns may hold anything (NaN canary) without affecting the output.  Every kernel runs to completion."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _shape(dtype):
    from paper_2605_02189_amd.synth_inputs import CONFIGS, StageShape
    if dtype == "fp32":
        return CONFIGS["C1"].with_(decode_steps=12)
    return StageShape("hz", 2, 512, 8, 2, 128, 1024, "bf16", 500000.0, 4, 6, 5, 90, 12)


def _run(shape, delays=None, canary=False, wb=0, flags=0):
    import torch
    from paper_2605_02189_amd.harness import StageRunner
    from paper_2605_02189_amd.synth_inputs import SynthInputs
    syn = SynthInputs(shape, seed=21, pool_elems=1 << 22, gain_jitter=0.1)
    run = StageRunner(shape, syn, wb_layers_per_copy=wb, flags=flags).load()
    st = run.stage
    if delays:
        st.debug_set_delays(*delays)
    if canary:
        st.debug_fill_free_gpu_pages(0x7FC0)
    run.warm_start()
    outs, keep = [], []
    for t in range(shape.decode_steps):
        mb = t % run.n
        hin = run.hidden_tensor(t, mb)
        hout = torch.empty_like(hin)
        keep.append(hin)            # a step is only enqueued: its input must stay alive until the final sync
        run.step(hin, hout)
        if canary and t % 3 == 2:
            st.debug_fill_free_gpu_pages(0x7FC0)          # synchronises, then poisons what is free now
        outs.append(hout)
    st.sync()
    outs = [o.cpu().view(torch.int16 if shape.dtype == "bf16" else torch.int32).numpy().copy() for o in outs]
    replica = []
    for mb in range(run.n):
        lens = st.get_ctx_lens(mb)
        for s in range(run.b_of[mb]):
            for l in range(shape.n_layers):
                K, V = st.kv_host_read(mb, s, l, 0, int(lens[s]))
                replica.append((K.copy(), V.copy()))
    stats = st.get_stats()
    st.destroy()
    return outs, replica, stats


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_injected_delays_change_nothing(dtype):
    shape = _shape(dtype)
    base_out, base_rep, _ = _run(shape)
    for delays, wb in (((20000, 0, 0), 0), ((0, 8000, 0), 1), ((0, 0, 8000), 1), ((3000, 3000, 3000), 0)):
        print("delays", delays, "wb_layers_per_copy", wb, flush=True)
        out, rep, stats = _run(shape, delays=delays, wb=wb)
        for t, (a, b) in enumerate(zip(out, base_out)):
            np.testing.assert_array_equal(a, b, err_msg=f"step {t} differs with delays {delays}")
        for (Ka, Va), (Kb, Vb) in zip(rep, base_rep):
            np.testing.assert_array_equal(Ka, Kb)
            np.testing.assert_array_equal(Va, Vb)
        assert stats["steps"] == shape.decode_steps


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_nan_canary_in_free_pages_never_reaches_the_output(dtype):
    shape = _shape(dtype)
    base_out, base_rep, _ = _run(shape)
    out, rep, _ = _run(shape, canary=True)
    for t, (a, b) in enumerate(zip(out, base_out)):
        np.testing.assert_array_equal(a, b, err_msg=f"step {t} differs with poisoned free pages")
    for (Ka, Va), (Kb, Vb) in zip(rep, base_rep):
        np.testing.assert_array_equal(Ka, Kb)
        np.testing.assert_array_equal(Va, Vb)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
def test_stream_ordered_evict_gives_the_same_results(dtype):
    """PIPEMAX_FLAG_STREAM_ORDERED_EVICT: the prefetch stream itself waits for the last reader of the pages it
    overwrites instead of the prefetch worker waiting on the host.  Same outputs and replica, also with every
    side path delayed and with the free pages poisoned (a copy that overtook its last reader, or a step that
    overtook its copy, would read the canary or stale bytes)."""
    from paper_2605_02189_amd import binding as pm
    shape = _shape(dtype)
    base_out, base_rep, _ = _run(shape)
    for delays, canary in ((None, False), ((6000, 3000, 3000), False), ((0, 0, 0), True), ((20000, 0, 0), True)):
        print("stream-ordered evict: delays", delays, "canary", canary, flush=True)
        out, rep, stats = _run(shape, delays=delays, canary=canary, flags=pm.FLAG_STREAM_ORDERED_EVICT)
        for t, (a, b) in enumerate(zip(out, base_out)):
            np.testing.assert_array_equal(a, b, err_msg=f"step {t} differs (delays {delays}, canary {canary})")
        for (Ka, Va), (Kb, Vb) in zip(rep, base_rep):
            np.testing.assert_array_equal(Ka, Kb)
            np.testing.assert_array_equal(Va, Vb)
        assert stats["steps"] == shape.decode_steps


def test_write_back_through_the_runtime_copy_equals_the_dma_engine_path(monkeypatch):
    """The worker thread copies a step's staged K,V rows to the host on a DMA engine (HSA runtime); when that path
    is refused -- forced here by the switch -- it falls back to the runtime's own copy.  Same bytes either way."""
    shape = _shape("bf16")
    base_out, base_rep, base_stats = _run(shape, wb=1)
    monkeypatch.setenv("PIPEMAX_NO_DMA_WRITEBACK", "1")
    out, rep, stats = _run(shape, wb=1)
    assert stats["d2h_bytes"] == base_stats["d2h_bytes"] > 0
    for t, (a, b) in enumerate(zip(out, base_out)):
        np.testing.assert_array_equal(a, b, err_msg=f"step {t}")
    for (Ka, Va), (Kb, Vb) in zip(rep, base_rep):
        np.testing.assert_array_equal(Ka, Kb)
        np.testing.assert_array_equal(Va, Vb)


def _run_scheduled(delays=None, canary=False):
    """Alg. 1 driving the stage (decode of a chosen part, releases, per-request prefetch) for 24 iterations."""
    import torch
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.harness import StageRunner
    from paper_2605_02189_amd.synth_inputs import StageShape, SynthInputs
    shape = StageShape("hzs", 2, 512, 8, 2, 128, 1024, "bf16", 500000.0, 4, 10, 5, 200, 24)
    syn = SynthInputs(shape, seed=23, pool_elems=1 << 22, gain_jitter=0.1)
    run = StageRunner(shape, syn, sigma=0.5, steps=24, gpu_pages=240).load()      # a tight pool: requests are released
    st = run.stage
    if delays:
        st.debug_set_delays(*delays)
    run.warm_start()
    sched = pm.Scheduler(alpha_s=4e-5, beta_s=2e-7, delta_s=1e-3, link_tokens_per_s=3.0e5, n_batches=4, window=4,
                         steady_rel_range=0.2, max_refine_steps=6)
    sched.attach(st)
    cur = torch.cuda.current_stream().cuda_stream
    outs, plans, keep = [], [], []
    for t in range(24):
        x = syn.hidden(t, 10)
        hin = torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).to("cuda:0")
        hout = torch.zeros_like(hin)
        keep.append(hin)            # the step is only enqueued: its input must outlive this loop iteration
        torch.cuda.synchronize()    # the fill of hout runs on torch's stream, the step on the library's
        d = sched.iterate(st, t, hin.data_ptr(), hout.data_ptr(), cur)
        if canary and t % 4 == 3:
            st.debug_fill_free_gpu_pages(0x7FC0)
        outs.append(hout[: d["n_exec"]])
        plans.append((d["exec"], d["prefetch"], d["evict"]))
    st.sync()
    outs = [o.cpu().view(torch.int16).numpy().copy() for o in outs]
    replica = []
    for mb in range(4):
        lens = st.get_ctx_lens(mb)
        for s in range(10):
            K, V = st.kv_host_read(mb, s, 1, 0, int(lens[s]))
            replica.append((K.copy(), V.copy()))
    sched.destroy()
    st.destroy()
    return outs, plans, replica


def test_scheduler_driven_iterations_are_immune_to_delays_and_poisoned_pages():
    base_out, base_plan, base_rep = _run_scheduled()
    assert any(p for _, p, _ in base_plan) and any(e for _, _, e in base_plan)
    for delays, canary in (((15000, 0, 0), False), ((0, 6000, 6000), False), ((2000, 2000, 2000), True)):
        print("delays", delays, "canary", canary, flush=True)
        out, plan, rep = _run_scheduled(delays, canary)
        assert plan == base_plan
        for t, (a, b) in enumerate(zip(out, base_out)):
            np.testing.assert_array_equal(a, b, err_msg=f"iteration {t} differs")
        for (Ka, Va), (Kb, Vb) in zip(rep, base_rep):
            np.testing.assert_array_equal(Ka, Kb)
            np.testing.assert_array_equal(Va, Vb)


def _run_prefill_then_decode(delays=None, canary=False):
    import torch
    from paper_2605_02189_amd.harness import StageRunner
    from paper_2605_02189_amd.synth_inputs import StageShape, SynthInputs
    shape = StageShape("hzp", 2, 512, 8, 2, 128, 1024, "bf16", 500000.0, 2, 24, 1, 70, 8)
    syn = SynthInputs(shape, seed=25, pool_elems=1 << 22, gain_jitter=0.1)
    ctx = {mb: syn.ctx_lens(mb).copy() for mb in range(2)}
    ctx[0][0] = 0
    run = StageRunner(shape, syn, sigma=1.0, steps=8 + 2 * 130, ctx_lens=ctx, gpu_pool_all_resident=True).load()
    st = run.stage
    if delays:
        st.debug_set_delays(*delays)
    cur = torch.cuda.current_stream().cuda_stream
    outs, keep = [], []
    st.prefetch_kv(0)
    for i, (seq, n_new) in enumerate(((0, 100), (1, 37), (0, 30))):          # chunks of 24 rows, fused path
        x = syn.hidden(100 + i, n_new)
        hin = torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).to("cuda:0")
        hout = torch.zeros_like(hin)
        keep.append(hin)
        torch.cuda.synchronize()
        st.prefill(0, seq, n_new, hin.data_ptr(), hout.data_ptr(), cur)
        if canary:
            st.debug_fill_free_gpu_pages(0x7FC0)
        outs.append(hout)
    # evict the prefilled batch (no copy: the replica must be complete), stream it back in, decode both batches
    st.evict_kv(0)
    run.warm_start()
    for t in range(8):
        mb = t % 2
        hin = run.hidden_tensor(t, mb)
        hout = torch.empty_like(hin)
        keep.append(hin)
        run.step(hin, hout)
        if canary and t % 3 == 2:
            st.debug_fill_free_gpu_pages(0x7FC0)
        outs.append(hout)
    st.sync()
    outs = [o.cpu().view(torch.int16).numpy().copy() for o in outs]
    st.destroy()
    return outs


def test_prefill_offload_and_later_decode_are_immune_to_delays_and_poisoned_pages():
    base = _run_prefill_then_decode()
    for delays, canary in (((0, 9000, 0), False), ((0, 0, 9000), False), ((4000, 4000, 4000), True)):
        print("delays", delays, "canary", canary, flush=True)
        out = _run_prefill_then_decode(delays, canary)
        for t, (a, b) in enumerate(zip(out, base)):
            np.testing.assert_array_equal(a, b, err_msg=f"output {t} differs")
