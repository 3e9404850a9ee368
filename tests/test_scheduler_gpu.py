"""The scheduler driving the real stage (pipemax_sched_iterate) against the scheduler oracle's counted
model (identical decisions, iteration by iteration) and the stage oracle (numerics of every executed
batch), plus the stage's own bookkeeping after each iteration."""
import numpy as np
import pytest

from conftest import rel_l2
from helpers import check_tables, make_oracle
from oracle import scheduler_oracle as so

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("static", [0, 900])
def test_scheduler_iterations_on_the_stage_match_both_oracles(static):
    import torch
    assert torch.cuda.is_available()
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.harness import StageRunner
    from paper_2605_02189_amd.synth_inputs import StageShape, SynthInputs
    shape = StageShape(name="sched", n_layers=2, hidden=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=2816,
                       dtype="bf16", rope_base=500000.0, n_microbatches=4, seqs_per_mb=12, ctx_lo=1, ctx_hi=260,
                       decode_steps=28)
    syn = SynthInputs(shape, seed=21, pool_elems=1 << 23, gain_jitter=0.1)
    ctx = {mb: syn.ctx_lens(mb).copy() for mb in range(4)}
    ctx[1][:3] = [15, 16, 32]                                  # page-boundary lengths among the candidates
    runner = StageRunner(shape, syn, sigma=0.5, steps=28, flags=pm.FLAG_CAPTURE_LAYERS, ctx_lens=ctx).load()
    st = runner.stage
    runner.warm_start()                                        # resident halves of every batch + all of D_0
    model = dict(alpha=4e-5, beta=2e-7, delta=1e-3, link_tokens_per_s=3.0e5)
    sched = pm.Scheduler(alpha_s=model["alpha"], beta_s=model["beta"], delta_s=model["delta"],
                         link_tokens_per_s=model["link_tokens_per_s"], n_batches=4, window=4, steady_rel_range=0.2,
                         max_refine_steps=6, refine_tol_s=model["alpha"] / 2, static_budget_tokens=static)
    sched.attach(st)
    lens = [st.get_ctx_lens(mb).tolist() for mb in range(4)]
    res = [(st.get_residency(mb) != 0).tolist() for mb in range(4)]
    sim = so.SchedulerSim(lens, res, st.get_stats()["gpu_pages_free"], window=4, rel_range=0.2, max_refine_steps=6,
                          refine_tol=model["alpha"] / 2, static_budget_tokens=static, **model)
    orc = make_oracle(shape, syn, runner.ctx0)
    cur = torch.cuda.current_stream().cuda_stream
    maxb = 12
    saw = dict(steady=False, evict=False, prefetch=False)
    for t in range(28):
        x = syn.hidden(t, maxb)
        hin = torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).to("cuda:0")
        hout = torch.zeros_like(hin)
        torch.cuda.synchronize()          # the fill runs on torch's stream, the step on the library's own
        got = sched.iterate(st, t, hin.data_ptr(), hout.data_ptr(), cur)
        want = sim.iterate(t)
        print(f"t {t} exec {got['exec']} prefetch {got['prefetch']} evict {got['evict']} budget "
              f"{got['budget_tokens']} steady {got['steady']}", flush=True)
        for key_g, key_w in (("exec", "exec"), ("prefetch", "prefetch"), ("evict", "evict")):
            assert got[key_g] == want[key_w], (t, key_g)
        assert (got["exec_batch"], got["prefetch_batch"], got["evict_batch"]) == \
               (want["exec_batch"], want["prefetch_batch"], want["evict_batch"])
        assert got["budget_tokens"] == want["budget"] and bool(got["steady"]) == want["steady"]
        assert got["t_hat_s"] == want["t_hat"] and got["n_exchanges"] == want["exchanges"]
        assert got["gpu_pages_free"] == want["gpu_pages_free"] == st.get_stats()["gpu_pages_free"]
        # numerics of the executed batch
        rows, mb = got["exec"], got["exec_batch"]
        if rows:
            ref_out, ref_layers = orc.decode_step(mb, syn.as_f32(x)[: len(rows)], seqs=rows)
            got_layers = st.get_layer_outputs(len(rows))
            for l in range(shape.n_layers):
                assert rel_l2(got_layers[l], ref_layers[l]) <= 1e-2, (t, l)
            assert rel_l2(hout[: len(rows)].float().cpu().numpy(), ref_out) <= 1e-2
        # the stage's bookkeeping equals the counted model's
        for m in range(4):
            assert st.get_ctx_lens(m).tolist() == sim.L[m]
            assert (st.get_residency(m) != 0).tolist() == sim.res[m]
        saw["steady"] |= want["steady"]
        saw["evict"] |= bool(want["evict"])
        saw["prefetch"] |= bool(want["prefetch"])
    assert saw["prefetch"] and saw["evict"]
    if not static:
        assert saw["steady"]
    st.sync()
    check_tables(runner)
    # the host replica holds every token: prompt bytes untouched, generated ones close to the oracle's
    for mb in range(4):
        for s in range(12):
            L0, L = int(runner.ctx0[mb][s]), int(sim.L[mb][s])
            for l in range(shape.n_layers):
                Kh, Vh = st.kv_host_read(mb, s, l, 0, L)
                K0, V0 = syn.kv_prefix(mb, s, l, L0)
                np.testing.assert_array_equal(Kh[:L0], K0)
                np.testing.assert_array_equal(Vh[:L0], V0)
                if L > L0:
                    Ko, Vo = orc.cached_kv(mb, s, l)
                    assert rel_l2(syn.as_f32(Kh[L0:]), Ko[L0:]) <= 1e-2
                    assert rel_l2(syn.as_f32(Vh[L0:]), Vo[L0:]) <= 1e-2
    sched.destroy()
    st.destroy()
