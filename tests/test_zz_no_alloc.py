"""pipemax_decode_step_noalloc (the entry point for callers that cannot allocate: its working buffers lie in the
library's static per-GPU scratch) against pipemax_decode_step on a twin stage with the same inputs: bit-identical
outputs, appended K,V and bookkeeping (both run the same kernels), on calls in a row that share the scratch: a
64-row and then a smaller 9-row micro-batch of one stage, then a 150-row pass of the large-tile path and a 20-row
one on another stage.  Oversized steps and the generic engine are refused with the stage unchanged."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _twin(shape, seed, ctx):
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.harness import StageRunner
    from paper_2605_02189_amd.synth_inputs import SynthInputs
    runs = []
    for _ in range(2):
        syn = SynthInputs(shape, seed=seed, pool_elems=1 << 23, gain_jitter=0.1)
        r = StageRunner(shape, syn, sigma=0.0, ctx_lens=ctx, gpu_pool_all_resident=True,
                        flags=pm.FLAG_CAPTURE_LAYERS).load()
        for mb in range(r.n):
            r.stage.prefetch_kv(mb)
        r.stage.sync()
        runs.append(r)
    return runs, syn


def _bits(t):
    import torch
    return t.cpu().view(torch.int16).numpy().copy()


def test_noalloc_step_equals_the_allocating_one_on_consecutive_calls_of_different_size():
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import StageShape
    cur = torch.cuda.current_stream().cuda_stream
    # stage A: fused path (64 rows, then 9); stage B: large-tile path (150 rows), then a 20-row micro-batch
    cases = [
        (StageShape("na", 2, 1024, 8, 2, 128, 2816, "bf16", 500000.0, 2, 64, 5, 700, 6),
         {0: None, 1: 9}, [0, 1, 0, 1]),
        (StageShape("nb", 1, 1024, 8, 2, 128, 2816, "bf16", 500000.0, 2, 150, 3, 90, 4),
         {0: None, 1: 20}, [0, 1, 1, 0]),
    ]
    for shape, cut, order in cases:
        from paper_2605_02189_amd.synth_inputs import SynthInputs
        syn0 = SynthInputs(shape, seed=31, pool_elems=1 << 23, gain_jitter=0.1)
        ctx = {mb: (syn0.ctx_lens(mb) if cut[mb] is None else syn0.ctx_lens(mb)[: cut[mb]]) for mb in range(2)}
        ctx[0][:3] = [15, 16, shape.ctx_hi]              # page-boundary lengths and the longest context
        (ref, new), syn = _twin(shape, 31, ctx)
        assert ref.stage.get_stats()["engine"] == 1
        for t, mb in enumerate(order):
            b = ref.b_of[mb]
            print(f"{shape.name}: call {t}, micro-batch {mb}, {b} rows", flush=True)
            hin = ref.hidden_tensor(t, mb)
            out_ref, out_new = torch.empty_like(hin), torch.empty_like(hin)
            ref.stage.decode_step(mb, hin.data_ptr(), out_ref.data_ptr(), cur)
            new.stage.decode_step_noalloc(mb, hin.data_ptr(), out_new.data_ptr(), cur)
            ref.stage.sync()
            new.stage.sync()
            np.testing.assert_array_equal(_bits(out_new), _bits(out_ref), err_msg=f"{shape.name} call {t}")
            np.testing.assert_array_equal(new.stage.get_layer_outputs(b), ref.stage.get_layer_outputs(b))
            assert np.isfinite(out_new.float().cpu().numpy()).all()
            np.testing.assert_array_equal(new.stage.get_ctx_lens(mb), ref.stage.get_ctx_lens(mb))
        for mb in range(2):                               # the appended K,V: device pages and host replica
            lens = ref.stage.get_ctx_lens(mb)
            for s in range(0, ref.b_of[mb], 7):
                for l in range(shape.n_layers):
                    L0, L = int(ctx[mb][s]), int(lens[s])
                    for fn in ("kv_dev_read", "kv_host_read"):
                        Ka, Va = getattr(new.stage, fn)(mb, s, l, L0, L - L0)
                        Kb, Vb = getattr(ref.stage, fn)(mb, s, l, L0, L - L0)
                        np.testing.assert_array_equal(Ka, Kb)
                        np.testing.assert_array_equal(Va, Vb)
        ref.stage.destroy()
        new.stage.destroy()


def test_noalloc_step_refuses_what_it_cannot_serve_and_changes_nothing():
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.harness import StageRunner
    from paper_2605_02189_amd.synth_inputs import CONFIGS, StageShape, SynthInputs
    cur = torch.cuda.current_stream().cuda_stream
    # (1) 256 rows at the 70B-shaped widths need more than the 64 MiB scratch (one layer, short prompts: small pools)
    big = CONFIGS["C4"].with_(n_layers=1, n_microbatches=1, ctx_lo=4, ctx_hi=4, decode_steps=2)
    # (2) the fp32 configuration runs on the generic engine
    for shape, code in ((big, pm.ERR_ARG), (CONFIGS["C1"].with_(n_microbatches=1), pm.ERR_STATE)):
        syn = SynthInputs(shape, seed=3, pool_elems=1 << 22)
        r = StageRunner(shape, syn, sigma=0.0, gpu_pool_all_resident=True)
        r.load_kv()
        r.stage.prefetch_kv(0)
        before = (r.stage.get_ctx_lens(0).copy(), r.stage.get_stats()["gpu_pages_free"])
        hin = r.hidden_tensor(0, 0)
        out = torch.empty_like(hin)
        with pytest.raises(pm.PipemaxError) as e:
            r.stage.decode_step_noalloc(0, hin.data_ptr(), out.data_ptr(), cur)
        assert e.value.code == code, e.value
        if code == pm.ERR_ARG:
            assert str(64 << 20) in str(e.value)
        np.testing.assert_array_equal(r.stage.get_ctx_lens(0), before[0])
        assert r.stage.get_stats()["gpu_pages_free"] == before[1]
        r.stage.decode_step(0, hin.data_ptr(), out.data_ptr(), cur)      # the stage still works
        r.stage.sync()
        assert np.isfinite(out.float().cpu().numpy()).all()
        r.stage.destroy()
