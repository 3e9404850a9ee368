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


def _run(shape, delays=None, canary=False, wb=0):
    import torch
    from paper_2605_02189_amd.harness import StageRunner
    from paper_2605_02189_amd.synth_inputs import SynthInputs
    syn = SynthInputs(shape, seed=21, pool_elems=1 << 22, gain_jitter=0.1)
    run = StageRunner(shape, syn, wb_layers_per_copy=wb).load()
    st = run.stage
    if delays:
        st.debug_set_delays(*delays)
    if canary:
        st.debug_fill_free_gpu_pages(0x7FC0)
    run.warm_start()
    outs = []
    for t in range(shape.decode_steps):
        mb = t % run.n
        hin = run.hidden_tensor(t, mb)
        hout = torch.empty_like(hin)
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
