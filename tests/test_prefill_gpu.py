"""Prefill through the C ABI against the stage oracle.  The oracle's definition of prefill is the
definition of causal attention: feeding the new tokens one at a time (its incremental decode is pinned
against a full causal recompute in tests/test_oracle_pins.py).  Bars as for decode: rel L2 <= 1e-5 (fp32),
<= 1e-2 (bf16) on the stage output of every chunk of rows, host replica == device pages byte for byte,
prompt bytes untouched, generated K/V close to the oracle's."""
import numpy as np
import pytest

from conftest import rel_l2
from helpers import check_tables, make_oracle

pytestmark = pytest.mark.gpu


def _hidden(torch, syn, shape, step, rows):
    x = syn.hidden(step, rows)
    if shape.dtype == "bf16":
        return x, torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16).to("cuda:0")
    return x, torch.from_numpy(np.array(x, dtype=np.float32)).to("cuda:0")


def _oracle_prefill(orc, syn, mb, seq, x):
    """Token by token: row t sees the cache plus rows <= t."""
    out = np.empty_like(syn.as_f32(x))
    xf = syn.as_f32(x)
    for t in range(xf.shape[0]):
        o, _ = orc.decode_step(mb, xf[t:t + 1], seqs=[seq])
        out[t] = o[0]
    return out


@pytest.mark.parametrize("case", ["mfma_fused_chunks", "mfma_wide_chunks", "mfma_xl_chunks", "mfma_xxl_chunks", "mfma_xl_wide_ffn",
                                  "mfma_xl_grouped",
                                  "mfma_long_context",
                                  "generic_fp32"])
def test_prefill_matches_token_by_token_oracle(case):
    import torch
    assert torch.cuda.is_available()
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.harness import StageRunner
    from paper_2605_02189_amd.synth_inputs import CONFIGS, StageShape, SynthInputs
    max_rows = None
    if case == "generic_fp32":
        shape = CONFIGS["C1"].with_(n_microbatches=1, seqs_per_mb=6)
        tol, plan = 1e-5, [(0, 21), (1, 19), (0, 8)]
    else:
        xl = case in ("mfma_xl_chunks", "mfma_xxl_chunks", "mfma_xl_wide_ffn", "mfma_xl_grouped")
        b = 70 if case == "mfma_wide_chunks" else 6 if xl else 20
        max_rows = 600 if xl else None                            # two 256-row blocks + a remainder per pass
        if case == "mfma_xxl_chunks":
            max_rows = 1300                                       # five 256-row blocks + 20 rows: beyond 1024 rows per pass
        # the wide FFN makes the gate/up GEMM of a 600-row pass un-split: SwiGLU runs in its epilogue
        if case == "mfma_xl_grouped":
            # every matrix has a multiple of 8 column blocks of 256: the large GEMM walks its tiles XCD by XCD
            shape = StageShape(name=case, n_layers=2, hidden=2048, n_q_heads=12, n_kv_heads=2, head_dim=128, ffn=2048,
                               dtype="bf16", rope_base=500000.0, n_microbatches=1, seqs_per_mb=b, ctx_lo=1, ctx_hi=60,
                               decode_steps=1)
        else:
            shape = StageShape(name=case, n_layers=1 if case == "mfma_xl_wide_ffn" else 2, hidden=1024, n_q_heads=8,
                               n_kv_heads=2, head_dim=128, ffn=16384 if case == "mfma_xl_wide_ffn" else 2816,
                               dtype="bf16", rope_base=500000.0, n_microbatches=1, seqs_per_mb=b, ctx_lo=1, ctx_hi=60,
                               decode_steps=1)
        tol = 1e-2
        # (sequence, new tokens): several chunks each; sequence 1 continues an existing prefix
        plan = [(0, 45), (1, 30), (0, 17)] if b == 20 else [(0, 150), (1, 75)]
        if xl:
            plan = [(0, 700), (1, 300)]
        if case == "mfma_xxl_chunks":
            plan = [(0, 1400), (1, 100)]
        if case == "mfma_long_context":                    # beyond the chunk kernel's 256 pages: per-row kernel
            plan = [(1, 30), (0, 5)]
    syn = SynthInputs(shape, seed=31, pool_elems=1 << 23, gain_jitter=0.1)
    ctx = {0: syn.ctx_lens(0).copy()}
    ctx[0][0] = 0                                          # a fresh request
    ctx[0][1] = 4085 if case == "mfma_long_context" else 37    # a prefix ending inside a page
    total_new = sum(n for _, n in plan)
    runner = StageRunner(shape, syn, sigma=0.0, steps=total_new + 4, ctx_lens=ctx, gpu_pool_all_resident=True,
                         max_rows=max_rows).load()
    st = runner.stage
    assert st.get_stats()["engine"] == (0 if case == "generic_fp32" else 1)
    orc = make_oracle(shape, syn, runner.ctx0)
    cur = torch.cuda.current_stream().cuda_stream
    st.prefetch_kv(0)
    step = 0
    for seq, n_new in plan:
        x, hin = _hidden(torch, syn, shape, step, n_new)
        hout = torch.empty_like(hin)
        L0 = int(st.get_ctx_lens(0)[seq])
        print(f"{case}: prefill seq {seq} at {L0} + {n_new}", flush=True)
        st.prefill(0, seq, n_new, hin.data_ptr(), hout.data_ptr(), cur)
        ref = _oracle_prefill(orc, syn, 0, seq, x)
        got = hout.float().cpu().numpy()
        chunk = max_rows or shape.seqs_per_mb
        for r0 in range(0, n_new, chunk):
            assert rel_l2(got[r0:r0 + chunk], ref[r0:r0 + chunk]) <= tol, (seq, r0)
        # a single row must also hold the bar (the last one sees the longest context)
        assert rel_l2(got[-1], ref[-1]) <= 2 * tol
        lens = st.get_ctx_lens(0)
        assert int(lens[seq]) == L0 + n_new == orc.ctx_len(0, seq)
        step += 1
    # decode steps of the whole micro-batch after the prefills
    for _ in range(2):
        b = runner.b_of[0]
        x, hin = _hidden(torch, syn, shape, step, b)
        hout = torch.empty_like(hin)
        st.decode_step(0, hin.data_ptr(), hout.data_ptr(), cur)
        ref, _ = orc.decode_step(0, syn.as_f32(x))
        assert rel_l2(hout.float().cpu().numpy(), ref) <= tol
        step += 1
    st.sync()
    check_tables(runner)
    lens = st.get_ctx_lens(0)
    for s in range(min(runner.b_of[0], 4)):
        L0, L = int(runner.ctx0[0][s]), int(lens[s])
        for l in range(shape.n_layers):
            Kh, Vh = st.kv_host_read(0, s, l, 0, L)
            Kd, Vd = st.kv_dev_read(0, s, l, 0, L)
            np.testing.assert_array_equal(Kd, Kh)
            np.testing.assert_array_equal(Vd, Vh)
            K0, V0 = syn.kv_prefix(0, s, l, L0)
            np.testing.assert_array_equal(Kh[:L0], K0)
            np.testing.assert_array_equal(Vh[:L0], V0)
            Ko, Vo = orc.cached_kv(0, s, l)
            assert rel_l2(syn.as_f32(Kh[L0:]), Ko[L0:]) <= tol
            assert rel_l2(syn.as_f32(Vh[L0:]), Vo[L0:]) <= tol
    # evict + prefetch brings the prefilled sequence back bit for bit, and the next step still matches
    st.evict_kv(0)
    st.prefetch_kv(0)
    b = runner.b_of[0]
    x, hin = _hidden(torch, syn, shape, step, b)
    hout = torch.empty_like(hin)
    st.decode_step(0, hin.data_ptr(), hout.data_ptr(), cur)
    ref, _ = orc.decode_step(0, syn.as_f32(x))
    assert rel_l2(hout.float().cpu().numpy(), ref) <= tol
    # error paths leave the lengths alone
    lens = st.get_ctx_lens(0).copy()
    x2 = torch.zeros(4, shape.hidden, dtype=runner.torch_dtype, device="cuda:0")
    st.sync()
    st.evict_kv(0, [2])
    for args, code in (((0, 2, 4), pm.ERR_NOT_RESIDENT), ((0, 99, 4), pm.ERR_ARG), ((0, 0, -1), pm.ERR_ARG),
                       ((0, 0, 10 ** 6), pm.ERR_STATE)):
        with pytest.raises(pm.PipemaxError) as e:
            st.prefill(*args, x2.data_ptr(), x2.data_ptr(), cur)
        assert e.value.code == code, args
    st.prefill(0, 0, 0, x2.data_ptr(), x2.data_ptr(), cur)
    np.testing.assert_array_equal(st.get_ctx_lens(0), lens)
    st.destroy()
