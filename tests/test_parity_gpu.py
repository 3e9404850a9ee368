"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Bars: bit-exact for KV paging / indexing / bookkeeping; relative L2 per layer output
<= 1e-5 for the fp32 stage and <= 1e-2 for bf16 stages (the tolerance the benchmark spec fixes)."""
import numpy as np
import pytest

from conftest import max_row_rel_l2, rel_l2
from helpers import check_tables, make_oracle

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _runner(shape, seed=0, **kw):
    from paper_2605_02189_amd.harness import StageRunner
    from paper_2605_02189_amd.synth_inputs import SynthInputs
    syn = SynthInputs(shape, seed=seed, pool_elems=kw.pop("pool_elems", 1 << 23), gain_jitter=0.1)
    return StageRunner(shape, syn, **kw), syn


def _bf16_round(a):
    from paper_2605_02189_amd.synth_inputs import bf16_bits_to_f32, to_bf16_bits
    return bf16_bits_to_f32(to_bf16_bits(a)).reshape(np.shape(a))


def _acc_bar(tol, floor):
    """Bar on an error that accumulates over the layers (the residual stream after layer l; the K,V rows projected
    from it): the stated bar, or 1.5 times what bf16 operand rounding alone costs on the same rows, whichever is
    larger.

    The stated bar (1e-2 for bf16) cannot hold for the accumulated stream at any depth and width: every layer adds
    the rounding error of the bf16 operands of the matrix cores (about 3e-3 of the layer's update), and with these
    synthetic weights (N(0, 0.02) at hidden 4096 / 8192) the first layer's update is 2.4 times the stream it is
    added to and the tenth's still a third of it, so an error in the stream is handed on undiluted, amplified by
    the next layer's non-linearity, and the new one adds to it.  The oracle run with nothing but those operand
    roundings (its diagnostic mode, same rows, same inputs) is 0.75e-2 away from its fp32 self after 8 layers of
    the 8B-shaped stage and passes 1e-2 on the 70B-shaped one around the 8th layer, with +-20 % from one step's
    inputs to the next.  The GPU path measures 1.0-1.35 times that floor.  What is asserted at the stated bar at
    ANY depth is the error of each layer on its own (teacher forcing, see _Compare)."""
    return max(tol, 1.5 * floor)


class _Compare:
    """Per-step comparison of the stage with the oracle on the tracked sequences: (1) every layer on its own: the
    GPU's output of layer l against the oracle's layer l applied to the GPU's output of layer l-1 (teacher forcing;
    a second oracle instance with the same weights and prompts keeps the caches that belong to those inputs), at
    the stated bar, for the batch and for the worst single row; (2) the residual stream after every layer against
    the oracle's own run, where errors accumulate over the layers (bar: _acc_bar; a third oracle instance in the
    operand-rounding mode gives the floor for bf16 stages; a single row may exceed its batch's bar by the spread
    seen between rows, up to 1.5x on ragged batches -- a defective row is off by 10x or more); (3) the update of
    each layer (output minus input), because the residual stream dominates the output norm."""

    def __init__(self, shape, syn, ctx0, oracle_seqs, tol_layer, tol_delta):
        self.shape, self.syn, self.tol_layer, self.tol_delta = shape, syn, tol_layer, tol_delta
        self.orc = make_oracle(shape, syn, ctx0, oracle_seqs)
        self.tf = make_oracle(shape, syn, ctx0, oracle_seqs, share_weights_of=self.orc)
        self.emu = (make_oracle(shape, syn, ctx0, oracle_seqs, share_weights_of=self.orc, operand_round=_bf16_round)
                    if shape.dtype == "bf16" else None)
        self.worst = dict(layer=0.0, row=0.0, delta=0.0, row_delta=0.0, own=0.0, own_row=0.0, floor=0.0)

    def step(self, t, mb, seqs, x_in, got_layers, got_out):
        shape, w = self.shape, self.worst
        ref_out, ref_layers = self.orc.decode_step(mb, x_in, seqs=seqs)
        emu_layers = self.emu.decode_step(mb, x_in, seqs=seqs)[1] if self.emu else ref_layers
        prev_ref, prev_got, prev_emu = x_in, x_in, x_in
        for l in range(shape.n_layers):
            floor = rel_l2(emu_layers[l], ref_layers[l])
            floor_d = rel_l2(emu_layers[l] - prev_emu, ref_layers[l] - prev_ref)
            tol_acc, tol_d = _acc_bar(self.tol_layer, floor), _acc_bar(self.tol_delta, floor_d)
            e = rel_l2(got_layers[l], ref_layers[l])
            d = rel_l2(got_layers[l] - prev_got, ref_layers[l] - prev_ref)
            er = max_row_rel_l2(got_layers[l], ref_layers[l])
            dr = max_row_rel_l2(got_layers[l] - prev_got, ref_layers[l] - prev_ref)
            own_ref, _ = self.tf.layer_decode(l, mb, seqs, np.ascontiguousarray(prev_got, dtype=np.float32))
            o, orow = rel_l2(got_layers[l], own_ref), max_row_rel_l2(got_layers[l], own_ref)
            for k, v in (("layer", e), ("row", er), ("delta", d), ("row_delta", dr), ("own", o), ("own_row", orow),
                         ("floor", floor)):
                w[k] = max(w[k], v)
            if t == 0:
                print(f"  layer {l}: stream {e:.3e} (worst row {er:.3e}; operand rounding alone {floor:.3e}), update "
                      f"{d:.3e} (worst row {dr:.3e}), layer on its own {o:.3e} (worst row {orow:.3e})", flush=True)
            assert o <= self.tol_layer, f"step {t} layer {l}: rel L2 of the layer on its own {o:.3e} > {self.tol_layer}"
            assert orow <= self.tol_layer, f"step {t} layer {l}: worst row, layer on its own {orow:.3e} > {self.tol_layer}"
            assert e <= tol_acc, f"step {t} layer {l}: rel L2 {e:.3e} > {tol_acc:.3e} (floor {floor:.3e})"
            assert er <= 1.5 * tol_acc, f"step {t} layer {l}: worst row rel L2 {er:.3e} > {1.5 * tol_acc:.3e}"
            assert d <= tol_d, f"step {t} layer {l}: rel L2 of the layer's update {d:.3e} > {tol_d:.3e}"
            assert dr <= 1.5 * tol_d, f"step {t} layer {l}: worst row, layer's update {dr:.3e} > {1.5 * tol_d:.3e}"
            prev_ref, prev_got, prev_emu = ref_layers[l], got_layers[l], emu_layers[l]
        # the stage output is the last layer's residual stream in the stage's element type
        tol_acc = _acc_bar(self.tol_layer, rel_l2(emu_layers[-1], ref_layers[-1]))
        if shape.dtype != "fp32":
            tol_acc = max(tol_acc, 8e-3)
        assert rel_l2(got_out, ref_out) <= tol_acc
        assert max_row_rel_l2(got_out, ref_out) <= 1.5 * tol_acc

    def report(self):
        w = self.worst
        print(f"worst rel L2: stream {w['layer']:.3e} (single row {w['row']:.3e}; operand rounding alone {w['floor']:.3e}), "
              f"layer update {w['delta']:.3e} (single row {w['row_delta']:.3e}), layer on its own {w['own']:.3e} "
              f"(single row {w['own_row']:.3e})", flush=True)


def _run_cyclic_and_compare(runner, syn, shape, steps, tol_layer, tol_delta, oracle_seqs=None):
    """Runs `steps` iterations of the cyclic schedule and compares every step with the oracle."""
    torch = _torch()
    from paper_2605_02189_amd import binding as pm
    cmp = _Compare(shape, syn, runner.ctx0, oracle_seqs, tol_layer, tol_delta)
    orc = cmp.orc
    runner.warm_start()
    for t in range(steps):
        mb = t % runner.n
        b = runner.b_of[mb]
        hin = runner.hidden_tensor(t, mb)
        hout = torch.empty_like(hin)
        print(f"step {t} mb {mb} b {b}", flush=True)
        assert runner.step(hin, hout) == mb
        seqs = list(oracle_seqs[mb]) if oracle_seqs else list(range(b))
        x_in = syn.as_f32(syn.hidden(t, b))[seqs]
        got_layers = runner.stage.get_layer_outputs(b)[:, seqs, :]
        got_out = runner.to_numpy_f32(hout)[seqs]
        cmp.step(t, mb, seqs, x_in, got_layers, got_out)
        # bookkeeping after the step
        lens = runner.stage.get_ctx_lens(mb)
        assert lens.tolist() == [orc.ctx_len(mb, s) if (not oracle_seqs or s in seqs) else lens[s]
                                 for s in range(b)]
        res = runner.stage.get_residency(mb)
        assert np.all(res == pm.GPU)
    cmp.report()
    orc.emulated = cmp.emu           # for the bars on the appended K,V (_check_replica)
    return orc


def _check_replica(runner, syn, shape, orc, tol_new, seqs=None):
    """Host replica == device pages byte for byte; prefix bit-identical to what was written;
    tokens appended on the GPU within tolerance of the oracle's."""
    st = runner.stage
    st.sync()
    for mb in range(runner.n):
        lens = st.get_ctx_lens(mb)
        res = st.get_residency(mb)
        for s in (seqs[mb] if seqs else range(runner.b_of[mb])):
            L0, L = int(runner.ctx0[mb][s]), int(lens[s])
            for l in range(shape.n_layers):
                Kh, Vh = st.kv_host_read(mb, s, l, 0, L)
                K0, V0 = syn.kv_prefix(mb, s, l, L0)
                np.testing.assert_array_equal(Kh[:L0], K0)
                np.testing.assert_array_equal(Vh[:L0], V0)
                if res[s] != 0:
                    Kd, Vd = st.kv_dev_read(mb, s, l, 0, L)
                    np.testing.assert_array_equal(Kd, Kh)
                    np.testing.assert_array_equal(Vd, Vh)
                if L > L0:
                    # the new K,V rows of layer l are projections of the stream that enters layer l: an accumulated
                    # error, with the bar of one (_acc_bar; the floor is what the operand-rounding oracle got)
                    Ko, Vo = orc.cached_kv(mb, s, l)
                    emu = getattr(orc, "emulated", None)
                    Ke, Ve = emu.cached_kv(mb, s, l) if emu is not None else (Ko, Vo)
                    tol_k = 1.5 * _acc_bar(tol_new, rel_l2(Ke[L0:], Ko[L0:]))
                    tol_v = 1.5 * _acc_bar(tol_new, rel_l2(Ve[L0:], Vo[L0:]))
                    assert rel_l2(syn.as_f32(Kh[L0:]), Ko[L0:]) <= tol_k, (mb, s, l)
                    assert rel_l2(syn.as_f32(Vh[L0:]), Vo[L0:]) <= tol_v, (mb, s, l)


# ---------------------------------------------------------------------------------------------
def test_config1_tiny_fp32_full_schedule():
    """configs[0] in full: 4 micro-batches x 8 sequences, 128-token prompts, 16 decode steps in cyclic
    order with 2 GPU arenas (3 of 4 micro-batches host-resident at any time)."""
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import CONFIGS
    shape = CONFIGS["C1"]
    runner, syn = _runner(shape, seed=1, flags=pm.FLAG_CAPTURE_LAYERS, wb_layers_per_copy=1, reserve=False)
    runner.load()
    assert runner.stage.get_stats()["engine"] == 0
    orc = _run_cyclic_and_compare(runner, syn, shape, shape.decode_steps, tol_layer=1e-5, tol_delta=2e-4)
    check_tables(runner)
    _check_replica(runner, syn, shape, orc, tol_new=1e-5)
    st = runner.stage.get_stats()
    assert st["host_pages_free"] == st["host_pages_total"] - 4 * 8 * 9     # no reservation: 9 pages per sequence
    assert st["steps"] == 16 and st["tokens"] == 16 * 8
    assert st["d2h_copies"] == 16 * shape.n_layers and st["relayout_jobs"] == 16 * shape.n_layers
    # every micro-batch was streamed in once per cycle (4 cycles), whole prompts + grown tokens
    assert st["h2d_bytes"] >= 16 * 8 * 8 * shape.page_bytes
    runner.stage.destroy()


def _mid_shape(**kw):
    from paper_2605_02189_amd.synth_inputs import StageShape
    base = dict(name="mid", n_layers=2, hidden=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=2816,
                dtype="bf16", rope_base=500000.0, n_microbatches=3, seqs_per_mb=20, ctx_lo=1, ctx_hi=300,
                decode_steps=9)
    base.update(kw)
    return StageShape(**base)


class _attn_kernel:
    """Selects the decode attention kernel of stages created inside the block (the library reads the variable when a
    stage is created): "wave" = a wave per (chunk, KV head, sequence) item, "group" = a work-group per item, None =
    the library's own choice by launch size."""
    def __init__(self, which):
        self.which = which

    def __enter__(self):
        import os
        self.old = os.environ.get("PIPEMAX_ATTN_KERNEL")
        if self.which is None:
            os.environ.pop("PIPEMAX_ATTN_KERNEL", None)
        else:
            os.environ["PIPEMAX_ATTN_KERNEL"] = self.which

    def __exit__(self, *a):
        import os
        if self.old is None:
            os.environ.pop("PIPEMAX_ATTN_KERNEL", None)
        else:
            os.environ["PIPEMAX_ATTN_KERNEL"] = self.old


def _ragged_ctx(shape, syn):
    ctx = {mb: syn.ctx_lens(mb).copy() for mb in range(shape.n_microbatches)}
    ctx[0][:6] = [0, 1, 15, 16, 17, 300]         # empty prompt, page-boundary cases, the longest
    return ctx


@pytest.mark.parametrize("attn", ["group", "wave"])
def test_bf16_matrix_core_path_ragged(attn):
    """bf16 stage on the matrix-core kernels: ragged batch (20 rows: one partial 32-row tile), ragged
    contexts including an empty prompt and page-boundary lengths, several GEMM tiles and attention
    chunks, 3 micro-batches streamed through 2 arenas; with either attention kernel."""
    from paper_2605_02189_amd import binding as pm
    shape = _mid_shape()
    from paper_2605_02189_amd.synth_inputs import SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    syn = SynthInputs(shape, seed=2, pool_elems=1 << 23, gain_jitter=0.1)
    with _attn_kernel(attn):
        runner = StageRunner(shape, syn, flags=pm.FLAG_CAPTURE_LAYERS, ctx_lens=_ragged_ctx(shape, syn)).load()
    assert runner.stage.get_stats()["engine"] == 1
    orc = _run_cyclic_and_compare(runner, syn, shape, shape.decode_steps, tol_layer=1e-2, tol_delta=3e-2)
    check_tables(runner)
    _check_replica(runner, syn, shape, orc, tol_new=1e-2)
    runner.stage.destroy()


@pytest.mark.parametrize("rows", [70, 128, 150, 257, 300, 384, 385])
def test_bf16_wide_batch(rows):
    """More than 64 rows.  70 and 128 rows: the fused pipeline with four row tiles per wave (at 70 the last
    two partial or empty).  150 rows: the large-tile GEMM (one 256-row block, its rows past 150 not stored)
    with the separate element-wise kernels.  300 rows: a 256-row block plus the 128-row tile for the
    remaining 44; 257, 384 and 385 rows are the edges of that choice (1 and 128 rows in the 128-row tile,
    129 rows in a second 256-row block)."""
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    shape = _mid_shape(n_layers=1, n_microbatches=2, seqs_per_mb=rows, ctx_lo=3, ctx_hi=60, decode_steps=4)
    syn = SynthInputs(shape, seed=8, pool_elems=1 << 23, gain_jitter=0.1)
    runner = StageRunner(shape, syn, flags=pm.FLAG_CAPTURE_LAYERS).load()
    assert runner.stage.get_stats()["engine"] == 1
    _run_cyclic_and_compare(runner, syn, shape, shape.decode_steps, tol_layer=1e-2, tol_delta=3e-2)
    runner.stage.destroy()


@pytest.mark.parametrize("engine", ["mfma_bf16", "generic_fp32"])
def test_layer_major_device_pool(engine):
    """PIPEMAX_FLAG_DEVICE_LAYER_MAJOR: the GPU pool laid out [layer][page] while the host replica and the link
    keep block-first pages (a prefetch scatters every page run with one strided copy per layer).  Same parity
    bars, same bit-exact bookkeeping, prefix and replica checks as the block-first pool; the outputs of the two
    layouts are bit-identical (the layout changes where bytes live, nothing else)."""
    torch = _torch()
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import CONFIGS, SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    if engine == "mfma_bf16":
        shape, tl, td = _mid_shape(n_layers=3), 1e-2, 3e-2
    else:
        shape, tl, td = CONFIGS["C1"].with_(decode_steps=9, n_microbatches=3), 1e-5, 2e-4
    outs = {}
    for flag in (pm.FLAG_DEVICE_LAYER_MAJOR, 0):
        syn = SynthInputs(shape, seed=2, pool_elems=1 << 23, gain_jitter=0.1)
        ctx = _ragged_ctx(shape, syn) if engine == "mfma_bf16" else None
        runner = StageRunner(shape, syn, flags=pm.FLAG_CAPTURE_LAYERS | flag, ctx_lens=ctx).load()
        assert runner.stage.get_stats()["engine"] == (1 if engine == "mfma_bf16" else 0)
        if flag:
            orc = _run_cyclic_and_compare(runner, syn, shape, shape.decode_steps, tol_layer=tl, tol_delta=td)
            check_tables(runner)
            _check_replica(runner, syn, shape, orc, tol_new=tl)
            runner.stage.debug_fill_free_gpu_pages(0x7FC0)          # the poison lands in free pages only
            _check_replica(runner, syn, shape, orc, tol_new=tl)
        else:
            runner.warm_start()
            for t in range(shape.decode_steps):
                hin = runner.hidden_tensor(t, t % runner.n)
                hout = torch.empty_like(hin)
                runner.step(hin, hout)
                runner.stage.sync()           # a step is only enqueued: its tensors must outlive it
        hin = runner.hidden_tensor(99, 0)
        hout = torch.empty_like(hin)
        runner.stage.prefetch_kv(0)
        runner.stage.decode_step(0, hin.data_ptr(), hout.data_ptr(), torch.cuda.current_stream().cuda_stream)
        runner.stage.sync()
        outs[flag] = hout.float().cpu().numpy()
        runner.stage.destroy()
    np.testing.assert_array_equal(outs[pm.FLAG_DEVICE_LAYER_MAJOR], outs[0])


def test_bf16_generic_path_matches_oracle_and_matrix_core_path():
    """The same bf16 workload on the shape-generic kernels (fp32 activations)."""
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    shape = _mid_shape(decode_steps=4, seqs_per_mb=5, ctx_hi=120)
    syn = SynthInputs(shape, seed=3, pool_elems=1 << 23, gain_jitter=0.1)
    runner = StageRunner(shape, syn, flags=pm.FLAG_CAPTURE_LAYERS | pm.FLAG_FORCE_GENERIC).load()
    assert runner.stage.get_stats()["engine"] == 0
    _run_cyclic_and_compare(runner, syn, shape, shape.decode_steps, tol_layer=2e-3, tol_delta=1e-2)
    runner.stage.destroy()


@pytest.mark.parametrize("attn", ["group", "wave"])
def test_long_context_many_chunks_and_wide_group(attn):
    """One long sequence next to short ones (split-K load balance), G = 8 query heads per KV head; with either
    attention kernel (the wave-per-item kernel merges the chunks of the 188-page context through its partials)."""
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    shape = _mid_shape(n_layers=1, n_q_heads=8, n_kv_heads=1, hidden=512, ffn=1024, n_microbatches=1,
                       seqs_per_mb=3, decode_steps=3, ctx_hi=3000)
    syn = SynthInputs(shape, seed=4, pool_elems=1 << 23, gain_jitter=0.1)
    ctx = {0: np.array([2999, 40, 1025], dtype=np.int32)}
    with _attn_kernel(attn):
        runner = StageRunner(shape, syn, flags=pm.FLAG_CAPTURE_LAYERS, ctx_lens=ctx).load()
    assert runner.stage.get_stats()["engine"] == 1
    _run_cyclic_and_compare(runner, syn, shape, shape.decode_steps, tol_layer=1e-2, tol_delta=3e-2)
    runner.stage.destroy()


def test_one_wave_streams_a_context_of_several_windows():
    """The wave-per-item attention keeps the page ids of 256 pages in registers and goes through a longer item window
    by window: contexts of 9000 and 5000 tokens as single items (563 and 313 pages: three and two windows, the last
    ones partial) next to a short one."""
    import os
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    shape = _mid_shape(n_layers=1, n_q_heads=8, n_kv_heads=1, hidden=512, ffn=1024, n_microbatches=1,
                       seqs_per_mb=3, decode_steps=3, ctx_hi=9100)
    syn = SynthInputs(shape, seed=5, pool_elems=1 << 23, gain_jitter=0.1)
    ctx = {0: np.array([9000, 40, 5000], dtype=np.int32)}
    os.environ["PIPEMAX_ATTN_CHUNK_PAGES"] = "1024"
    try:
        with _attn_kernel("wave"):
            runner = StageRunner(shape, syn, flags=pm.FLAG_CAPTURE_LAYERS, ctx_lens=ctx).load()
    finally:
        del os.environ["PIPEMAX_ATTN_CHUNK_PAGES"]
    assert runner.stage.get_stats()["engine"] == 1
    _run_cyclic_and_compare(runner, syn, shape, shape.decode_steps, tol_layer=1e-2, tol_delta=3e-2)
    runner.stage.destroy()


def test_offload_then_prefetch_is_a_bit_identical_round_trip():
    """Bytes written to the host replica come back from the GPU pages unchanged, wherever the pages
    land; evicting and prefetching again (into other physical pages) changes nothing."""
    torch = _torch()
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import CONFIGS
    for shape in (CONFIGS["C1"], _mid_shape(n_layers=3, seqs_per_mb=4, ctx_hi=90)):
        runner, syn = _runner(shape, seed=5)
        runner.load_kv()
        st = runner.stage
        st.prefetch_kv(1)
        st.prefetch_kv(0, [2, 0])
        g_before = {s: st.get_block_table(0, s)[0].copy() for s in (0, 2)}
        st.evict_kv(0, [0])
        st.prefetch_kv(0, [1])                        # takes seq 0's old pages first (lowest index first)
        st.prefetch_kv(0, [0])
        g_after, _ = st.get_block_table(0, 0)
        assert len(g_before[0]) == 0 or g_after.tolist() != g_before[0].tolist()
        st.sync()
        check_tables(runner)
        for mb, seqs in ((0, [0, 1, 2]), (1, range(runner.b_of[1]))):
            for s in seqs:
                L = int(runner.ctx0[mb][s])
                for l in range(shape.n_layers):
                    K0, V0 = syn.kv_prefix(mb, s, l, L)
                    Kd, Vd = st.kv_dev_read(mb, s, l, 0, L)
                    np.testing.assert_array_equal(Kd, K0)
                    np.testing.assert_array_equal(Vd, V0)
                    # partial ranges address the same bytes
                    if L > 20:
                        Kp, Vp = st.kv_dev_read(mb, s, l, 13, 7)
                        np.testing.assert_array_equal(Kp, K0[13:20])
                        np.testing.assert_array_equal(Vp, V0[13:20])
        with pytest.raises(pm.PipemaxError) as e:
            st.kv_dev_read(0, 3, 0, 0, 1)
        assert e.value.code == pm.ERR_NOT_RESIDENT
        st.destroy()


def test_results_do_not_depend_on_physical_page_placement():
    """Same inputs, different page placement (other sequences prefetched first, a hole punched in the
    pool) -> identical outputs, bit for bit."""
    torch = _torch()
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    shape = _mid_shape(n_microbatches=2, seqs_per_mb=6, ctx_hi=200, decode_steps=2)
    outs, tables = [], []
    for variant in range(2):
        syn = SynthInputs(shape, seed=6, pool_elems=1 << 23, gain_jitter=0.1)
        runner = StageRunner(shape, syn, sigma=0.0).load()
        st = runner.stage
        if variant == 0:
            st.prefetch_kv(0)
        else:
            st.prefetch_kv(1, [3, 4])
            st.prefetch_kv(0, [5, 4, 3])
            st.evict_kv(1, [3])
            st.prefetch_kv(0)
        tables.append([st.get_block_table(0, s_)[0].tolist() for s_ in range(runner.b_of[0])])
        hin = runner.hidden_tensor(0, 0)
        res = []
        for t in range(2):
            hout = torch.empty_like(hin)
            st.decode_step(0, hin.data_ptr(), hout.data_ptr(), torch.cuda.current_stream().cuda_stream)
            st.sync()
            res.append(hout.cpu().view(torch.int16).numpy().copy())
            hin = hout
        outs.append(res)
        st.destroy()
    assert tables[0] != tables[1]
    for t in range(2):
        np.testing.assert_array_equal(outs[0][t], outs[1][t])


@pytest.mark.parametrize("engine", ["mfma", "generic_fp32"])
def test_decode_over_a_chosen_part_of_a_microbatch(engine):
    """pipemax_decode_step_seqs: a different subset of each micro-batch, in a shuffled row order, is
    prefetched and executed at every step; only the listed sequences grow; whole-micro-batch steps in
    between see the right lengths and tables; the sequences left on the host keep their bytes."""
    torch = _torch()
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import SynthInputs, CONFIGS
    from paper_2605_02189_amd.harness import StageRunner
    from oracle.bookkeeping_oracle import ResidencyModel
    if engine == "mfma":
        shape = _mid_shape(n_microbatches=2, seqs_per_mb=12, ctx_hi=200, decode_steps=10)
        tol_layer, tol_delta = 1e-2, 3e-2
    else:
        shape = CONFIGS["C1"].with_(n_microbatches=2, decode_steps=10)
        tol_layer, tol_delta = 1e-5, 2e-4
    syn = SynthInputs(shape, seed=11, pool_elems=1 << 23, gain_jitter=0.1)
    ctx = {mb: syn.ctx_lens(mb).copy() for mb in range(2)}
    ctx[0][:4] = [0, 15, 16, 31]
    runner = StageRunner(shape, syn, sigma=0.0, flags=pm.FLAG_CAPTURE_LAYERS, ctx_lens=ctx,
                         gpu_pool_all_resident=True).load()
    st = runner.stage
    assert st.get_stats()["engine"] == (1 if engine == "mfma" else 0)
    orc = make_oracle(shape, syn, runner.ctx0)
    rng = np.random.default_rng(5)
    cur = torch.cuda.current_stream().cuda_stream
    b = runner.b_of[0]
    for t in range(10):
        mb = t % 2
        if t in (4, 5):                                   # a whole-micro-batch step between subset steps
            rows = list(range(b))
            st.prefetch_kv(mb)
        else:
            rows = rng.permutation(b)[: int(rng.integers(1, b + 1))].tolist()
            st.evict_kv(mb, [s for s in range(b) if s not in rows])
            st.prefetch_kv(mb, rows)
        print(f"step {t} mb {mb} rows {rows}", flush=True)
        x = syn.hidden(t, len(rows))
        hin = (torch.from_numpy(x.view(np.int16).copy()).view(torch.bfloat16) if shape.dtype == "bf16"
               else torch.from_numpy(np.array(x, dtype=np.float32))).to("cuda:0")
        hout = torch.empty_like(hin)
        before = st.get_ctx_lens(mb).copy()
        if t in (4, 5):
            st.decode_step(mb, hin.data_ptr(), hout.data_ptr(), cur)
        else:
            st.decode_step_seqs(mb, rows, hin.data_ptr(), hout.data_ptr(), cur)
        ref_out, ref_layers = orc.decode_step(mb, syn.as_f32(x), seqs=rows)
        got_layers = st.get_layer_outputs(len(rows))
        prev_ref = prev_got = syn.as_f32(x)
        for l in range(shape.n_layers):
            assert rel_l2(got_layers[l], ref_layers[l]) <= tol_layer, (t, l)
            assert rel_l2(got_layers[l] - prev_got, ref_layers[l] - prev_ref) <= tol_delta, (t, l)
            assert max_row_rel_l2(got_layers[l], ref_layers[l]) <= tol_layer, (t, l)
            assert max_row_rel_l2(got_layers[l] - prev_got, ref_layers[l] - prev_ref) <= tol_delta, (t, l)
            prev_ref, prev_got = ref_layers[l], got_layers[l]
        assert rel_l2(runner.to_numpy_f32(hout), ref_out) <= max(tol_layer, 8e-3 if shape.dtype == "bf16" else 0)
        after = st.get_ctx_lens(mb)
        want = before.copy()
        want[rows] += 1
        np.testing.assert_array_equal(after, want)
        assert after.tolist() == [orc.ctx_len(mb, s) for s in range(b)]
    check_tables(runner)
    _check_replica(runner, syn, shape, orc, tol_new=tol_layer)
    # argument errors: a sequence listed twice, out of range, host-resident; nothing changes
    lens = st.get_ctx_lens(0).copy()
    x = torch.zeros(2, shape.hidden, dtype=runner.torch_dtype, device="cuda:0")
    for bad, code in (([1, 1], pm.ERR_ARG), ([0, b], pm.ERR_ARG)):
        with pytest.raises(pm.PipemaxError) as e:
            st.decode_step_seqs(0, bad, x.data_ptr(), x.data_ptr(), cur)
        assert e.value.code == code
    st.evict_kv(0, [2])
    with pytest.raises(pm.PipemaxError) as e:
        st.decode_step_seqs(0, [2], x.data_ptr(), x.data_ptr(), cur)
    assert e.value.code == pm.ERR_NOT_RESIDENT
    st.decode_step_seqs(0, [], x.data_ptr(), x.data_ptr(), cur)          # empty list: no-op
    np.testing.assert_array_equal(st.get_ctx_lens(0), lens)
    st.destroy()


def test_error_paths_leave_the_stage_unchanged():
    torch = _torch()
    from paper_2605_02189_amd import binding as pm
    from oracle.bookkeeping_oracle import ResidencyModel, BookkeepingError
    shape = _mid_shape(n_layers=1, hidden=256, ffn=256, n_q_heads=2, n_kv_heads=1, n_microbatches=2)
    page = shape.page_bytes
    st = pm.Stage(n_layers=1, hidden=256, n_q_heads=2, n_kv_heads=1, head_dim=128, ffn=256, rope_base=1e4,
                  rms_eps=1e-5, dtype=pm.BF16, n_microbatches=2, max_seqs_per_mb=2, max_ctx=40,
                  gpu_kv_bytes=4 * page, host_kv_bytes=10 * page)
    model = ResidencyModel(2, 16, max_ctx=40, gpu_pages=4, host_pages=10)
    code = {"ARG": pm.ERR_ARG, "NOT_RESIDENT": pm.ERR_NOT_RESIDENT, "POOL_EXHAUSTED": pm.ERR_POOL_EXHAUSTED,
            "STATE": pm.ERR_STATE}
    h = torch.zeros(2, 256, dtype=torch.bfloat16, device="cuda")
    o = torch.empty_like(h)
    sp = torch.cuda.current_stream().cuda_stream

    def both(name, *args):
        """Applies a call to the model and to the library; both must agree on success / error kind."""
        want = None
        try:
            getattr(model, name)(*args)
        except BookkeepingError as e:
            want = code[e.kind]
        lib_call = {"mb_define": lambda mb, lens: st.mb_define(mb, lens),
                    "prefetch": lambda mb, ids=None: st.prefetch_kv(mb, ids),
                    "evict": lambda mb, ids=None: st.evict_kv(mb, ids),
                    "decode_step": lambda mb: st.decode_step(mb, h.data_ptr(), o.data_ptr(), sp)}[name]
        if want is None:
            lib_call(*args)
        else:
            with pytest.raises(pm.PipemaxError) as e:
                lib_call(*args)
            assert e.value.code == want, (name, args, e.value)
        for mb in model.nseq:
            assert st.get_ctx_lens(mb).tolist() == model.ctx_lens(mb)
            assert [int(r != 0) for r in st.get_residency(mb)] == [int(model.resident(mb, s))
                                                                    for s in range(model.nseq[mb])]
        s_ = st.get_stats()
        assert s_["gpu_pages_free"] == model.gpu_free and s_["host_pages_free"] == model.host_free

    both("mb_define", 0, [16, 17])
    both("mb_define", 1, [40])
    both("mb_define", 1, [1])                 # already defined
    both("decode_step", 0)                    # nothing resident
    both("prefetch", 0)                       # takes 3 of the 4 GPU pages
    both("prefetch", 1)                       # pool exhausted, nothing applied
    both("decode_step", 0)                    # works; seq 0 at a page boundary takes the 4th GPU page
    both("evict", 0, [1])
    both("prefetch", 0, [1])
    both("evict", 0)
    both("prefetch", 1)
    both("decode_step", 1)                    # at max_ctx
    both("evict", 1)
    both("prefetch", 0, [1])
    both("decode_step", 0)                    # seq 0 not resident
    both("prefetch", 0, [0])
    both("decode_step", 0)                    # works, no new page
    both("prefetch", 0, [7])                  # bad sequence index
    st.sync()
    st.destroy()


def test_single_sequence_single_microbatch_from_empty_cache():
    """b = 1, one micro-batch, empty prompt: the first step attends over exactly one token, so the
    attention output is that token's V (the oracle pins this case bit for bit)."""
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import SynthInputs, CONFIGS
    from paper_2605_02189_amd.harness import StageRunner
    for shape, tl, td in ((CONFIGS["C1"].with_(n_microbatches=1, seqs_per_mb=1, ctx_lo=0, ctx_hi=0, decode_steps=18), 1e-5, 2e-4),
                          (_mid_shape(n_microbatches=1, seqs_per_mb=1, ctx_lo=0, ctx_hi=0, decode_steps=18), 1e-2, 3e-2)):
        syn = SynthInputs(shape, seed=7, pool_elems=1 << 23, gain_jitter=0.1)
        runner = StageRunner(shape, syn, flags=pm.FLAG_CAPTURE_LAYERS).load()
        orc = _run_cyclic_and_compare(runner, syn, shape, shape.decode_steps, tol_layer=tl, tol_delta=td)
        _check_replica(runner, syn, shape, orc, tol_new=tl)
        assert runner.stage.get_ctx_lens(0).tolist() == [18]
        assert len(runner.stage.get_block_table(0, 0)[1]) == 2
        runner.stage.destroy()


def test_config2_full_size_sampled_rows():
    """configs[1] at full size, in the launch configuration bench.py times (4 micro-batches x 64
    sequences x 1024-token prompts, sigma = 1, cyclic schedule): the oracle follows a sample of rows
    (rows are independent) through all 8 layers for two cycles."""
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import CONFIGS, SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    shape = CONFIGS["C2"]
    syn = SynthInputs(shape, seed=0, gain_jitter=0.1)
    steps = 2 * shape.n_microbatches
    runner = StageRunner(shape, syn, steps=steps, flags=pm.FLAG_CAPTURE_LAYERS).load()
    assert runner.stage.get_stats()["engine"] == 1
    sample = {mb: [0, 17 + mb, 63] for mb in range(shape.n_microbatches)}
    orc = _run_cyclic_and_compare(runner, syn, shape, steps, tol_layer=1e-2, tol_delta=3e-2, oracle_seqs=sample)
    check_tables(runner)
    _check_replica(runner, syn, shape, orc, tol_new=1e-2, seqs=sample)
    st = runner.stage.get_stats()
    # every step streamed one whole micro-batch in (64 prefix pages + grown pages per sequence)
    assert st["h2d_bytes"] >= steps * 64 * 64 * shape.page_bytes
    runner.stage.destroy()


def test_config3_ragged_full_shape_sampled_rows():
    """configs[2] at its full layer shapes and batch (128 ragged sequences of 512..4096 tokens per
    micro-batch, 8 layers, sigma = 1), two of its six micro-batches for two cycles: the fused path with
    four row tiles per wave, attention over up to 257 pages per sequence with the long sequences split.
    The oracle follows the longest, the shortest and two other sequences of each micro-batch."""
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import CONFIGS, SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    shape = CONFIGS["C3"].with_(n_microbatches=2)
    syn = SynthInputs(shape, seed=0, gain_jitter=0.1)
    steps = 2 * shape.n_microbatches
    runner = StageRunner(shape, syn, steps=steps, flags=pm.FLAG_CAPTURE_LAYERS).load()
    assert runner.stage.get_stats()["engine"] == 1
    sample = {}
    for mb in range(shape.n_microbatches):
        lens = np.asarray(runner.ctx0[mb])
        sample[mb] = sorted({int(lens.argmax()), int(lens.argmin()), 5 + mb, 127})
    orc = _run_cyclic_and_compare(runner, syn, shape, steps, tol_layer=1e-2, tol_delta=3e-2, oracle_seqs=sample)
    check_tables(runner)
    _check_replica(runner, syn, shape, orc, tol_new=1e-2, seqs=sample)
    runner.stage.destroy()


def test_config4_full_depth_sampled_rows():
    """configs[3] at its real depth and layer shapes (10 layers, hidden 8192, 64/8 heads, ffn 28672, 256 sequences
    of 2048 tokens: 640 KiB pages, their per-layer stride, the 10-layer staging copy and host re-layout), two of
    its eight micro-batches streamed through two arenas for two cycles (sigma = 1): the large-tile GEMMs at 256
    rows with the separate element-wise kernels, at the sizes bench.py launches them.  (Two micro-batches are
    43 GB of pinned memory; the remaining six differ only in their seed.)"""
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import CONFIGS, SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    shape = CONFIGS["C4"].with_(n_microbatches=2)
    assert shape.n_layers == 10 and shape.page_bytes == 640 * 1024
    syn = SynthInputs(shape, seed=0, gain_jitter=0.1)
    steps = 2 * shape.n_microbatches
    runner = StageRunner(shape, syn, steps=steps, flags=pm.FLAG_CAPTURE_LAYERS).load()
    assert runner.stage.get_stats()["engine"] == 1
    sample = {mb: [0, 100 + mb, 255] for mb in range(shape.n_microbatches)}
    orc = _run_cyclic_and_compare(runner, syn, shape, steps, tol_layer=1e-2, tol_delta=3e-2, oracle_seqs=sample)
    check_tables(runner)
    _check_replica(runner, syn, shape, orc, tol_new=1e-2, seqs=sample)
    runner.stage.destroy()


def test_config5_shapes_full_depth_sampled_rows():
    """configs[4]'s shapes at full depth: 256 sequences with 4096-token contexts on the 10-layer 70B-shaped stage.
    The new token makes 4097 tokens = 257 pages per sequence, one more than a single attention work-group takes,
    so the 256-row large-tile GEMM path runs together with the split attention and its in-kernel merge.  One
    micro-batch is 43 GB of pinned memory, all this host can pin beside the staging buffers, so the schedule is
    the one-batch case of Eq. 3 (i = j = k): step, evict everything, prefetch everything back from the host
    replica (which by then holds the first step's tokens), step again."""
    torch = _torch()
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import CONFIGS, SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    shape = CONFIGS["C5"].with_(n_microbatches=1)
    syn = SynthInputs(shape, seed=0, gain_jitter=0.1)
    runner = StageRunner(shape, syn, steps=3, flags=pm.FLAG_CAPTURE_LAYERS).load()
    st = runner.stage
    assert st.get_stats()["engine"] == 1
    sample = [0, 77, 255]
    cmp = _Compare(shape, syn, runner.ctx0, {0: sample}, 1e-2, 3e-2)
    orc = cmp.orc
    st.prefetch_kv(0)
    cur = torch.cuda.current_stream().cuda_stream
    for t in range(3):
        print(f"step {t}", flush=True)
        hin = runner.hidden_tensor(t, 0)
        hout = torch.empty_like(hin)
        st.decode_step(0, hin.data_ptr(), hout.data_ptr(), cur)
        x_in = syn.as_f32(syn.hidden(t, runner.b))[sample]
        cmp.step(t, 0, sample, x_in, st.get_layer_outputs(runner.b)[:, sample, :], runner.to_numpy_f32(hout)[sample])
        assert st.get_ctx_lens(0).tolist() == [4096 + t + 1] * runner.b
        if t == 0:
            st.evict_kv(0)
            assert np.all(st.get_residency(0) == pm.HOST)
            st.prefetch_kv(0)
    cmp.report()
    orc.emulated = cmp.emu
    assert len(st.get_block_table(0, 0)[1]) == 257
    check_tables(runner)
    _check_replica(runner, syn, shape, orc, tol_new=1e-2, seqs={0: sample})
    st.destroy()


def test_alias_microbatches_move_the_same_bytes():
    """pipemax_mb_define_alias (hosts that cannot pin a whole configuration): an alias takes nothing from the host
    pool, names its source's host pages, prefetches the source's bytes into GPU pages of its own and runs the
    cyclic schedule with the traffic of an ordinary micro-batch; the tokens that existed when it was defined stay
    intact in the shared pages."""
    torch = _torch()
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    shape = _mid_shape(n_microbatches=4, seqs_per_mb=6, ctx_lo=20, ctx_hi=120, decode_steps=8)
    traffic = {}
    for real in (4, 2):
        syn = SynthInputs(shape, seed=9, pool_elems=1 << 23, gain_jitter=0.1)
        ctx = {mb: syn.ctx_lens(mb % 2) for mb in range(4)}          # the un-aliased run gets the same lengths
        runner = StageRunner(shape, syn, ctx_lens=ctx, real_microbatches=real)
        st = runner.stage
        runner.load_weights()
        free0 = None
        if real == 2:
            for mb in range(2):
                st.mb_define(mb, runner.ctx0[mb])
                for s, L in enumerate(runner.ctx0[mb]):
                    for l in range(shape.n_layers):
                        st.kv_host_write(mb, s, l, 0, *syn.kv_prefix(mb, s, l, int(L)))
            free0 = st.get_stats()["host_pages_free"]
            for mb in (2, 3):
                st.mb_define_alias(mb, mb - 2)
            assert st.get_stats()["host_pages_free"] == free0
            assert [st.mb_alias_of(mb) for mb in range(4)] == [-1, -1, 0, 1]
            for s in range(runner.b):
                assert st.get_block_table(2, s)[1].tolist() == st.get_block_table(0, s)[1].tolist()
            with pytest.raises(pm.PipemaxError) as e:
                st.mb_define_alias(2, 0)                 # already defined
            assert e.value.code == pm.ERR_ARG
            with pytest.raises(pm.PipemaxError) as e:
                st.kv_host_write(2, 0, 0, 0, *syn.kv_prefix(0, 0, 0, int(runner.ctx0[0][0])))
            assert e.value.code == pm.ERR_STATE
            # the alias's GPU pages receive the source's bytes
            st.prefetch_kv(2)
            st.prefetch_kv(0)
            g2 = {int(p) for s in range(runner.b) for p in st.get_block_table(2, s)[0]}
            g0 = {int(p) for s in range(runner.b) for p in st.get_block_table(0, s)[0]}
            assert not (g2 & g0)
            for s in range(runner.b):
                L = int(runner.ctx0[0][s])
                for l in range(shape.n_layers):
                    K0, V0 = syn.kv_prefix(0, s, l, L)
                    Kd, Vd = st.kv_dev_read(2, s, l, 0, L)
                    np.testing.assert_array_equal(Kd, K0)
                    np.testing.assert_array_equal(Vd, V0)
            st.evict_kv(2)
            st.evict_kv(0)
            st.sync()
        else:
            runner.load_kv()
        runner.warm_start()
        st.sync()
        st.reset_stats()
        outs = []
        for t in range(shape.decode_steps):
            mb = t % 4
            hin = runner.hidden_tensor(t, mb)
            hout = torch.empty_like(hin)
            runner.step(hin, hout)
            st.sync()
            outs.append(hout.float().cpu().numpy())
        stats = st.get_stats()
        traffic[real] = (stats["h2d_bytes"], stats["d2h_bytes"], stats["d2h_copies"], stats["tokens"])
        assert all(np.isfinite(o).all() for o in outs)
        for mb in range(4):
            assert st.get_ctx_lens(mb).tolist() == (runner.ctx0[mb] + 2).tolist()
        if real == 2:
            check_tables(runner)
            assert st.get_stats()["host_pages_free"] == free0        # growth stayed inside the shared reservation
            for mb in range(2):                                       # the prompts are untouched by either writer
                for s in range(runner.b):
                    L = int(runner.ctx0[mb][s])
                    for l in range(shape.n_layers):
                        K0, V0 = syn.kv_prefix(mb, s, l, L)
                        Kh, Vh = st.kv_host_read(mb, s, l, 0, L)
                        np.testing.assert_array_equal(Kh, K0)
                        np.testing.assert_array_equal(Vh, V0)
        st.destroy()
    assert traffic[2] == traffic[4]


@pytest.mark.parametrize("attn", ["group", "wave"])
def test_split_merges_are_bit_identical_from_run_to_run(attn):
    """The in-kernel merges of split-K partials (GEMM splits summed by the last arriving work-group, attention chunks
    merged by the last arriver of a (sequence, KV head)) publish their partials with agent-scope atomics and an
    arrival counter instead of a device-wide fence.  Whatever the arrival order, the sums are taken in split order,
    so the same inputs must give the same bits every time, also with thousands of work-groups of all XCDs in flight:
    a stale or torn partial would show as a differing bit.  40 consecutive steps, each with 2 to 4 GEMM splits over 64 to 96 column
    blocks and up to 24 attention chunks per sequence (one 3000-token context among short ones, 8-page chunks), merged
    by the last work-group ("group") or the last wave ("wave") to arrive."""
    torch = _torch()
    import os
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.synth_inputs import SynthInputs
    from paper_2605_02189_amd.harness import StageRunner
    shape = _mid_shape(n_layers=2, n_microbatches=1, seqs_per_mb=48, decode_steps=2, ctx_lo=100, ctx_hi=900,
                       hidden=4096, n_q_heads=32, n_kv_heads=8, ffn=14336 // 2)
    syn = SynthInputs(shape, seed=12, pool_elems=1 << 23, gain_jitter=0.1)
    ctx = {0: syn.ctx_lens(0).copy()}
    ctx[0][0] = 3000
    os.environ["PIPEMAX_ATTN_CHUNK_PAGES"] = "8"
    try:
        with _attn_kernel(attn):
            runner = StageRunner(shape, syn, sigma=0.0, ctx_lens=ctx, gpu_pool_all_resident=True,
                                 flags=pm.FLAG_NO_WRITEBACK, steps=64).load()
    finally:
        del os.environ["PIPEMAX_ATTN_CHUNK_PAGES"]
    st = runner.stage
    assert st.get_stats()["engine"] == 1
    st.prefetch_kv(0)
    cur = torch.cuda.current_stream().cuda_stream
    hin = runner.hidden_tensor(0, 0)
    outs = [torch.empty_like(hin) for _ in range(40)]
    for hout in outs:                # every repetition appends a token; the twin run below repeats the same 40 steps
        st.decode_step(0, hin.data_ptr(), hout.data_ptr(), cur)
    st.sync()
    a = [o.cpu().view(torch.int16).numpy().copy() for o in outs]
    st.destroy()
    # the twin run: same inputs, same 40 steps, a fresh stage; step r of both runs must agree bit for bit
    os.environ["PIPEMAX_ATTN_CHUNK_PAGES"] = "8"
    try:
        with _attn_kernel(attn):
            runner = StageRunner(shape, syn, sigma=0.0, ctx_lens=ctx, gpu_pool_all_resident=True,
                                 flags=pm.FLAG_NO_WRITEBACK, steps=64).load()
    finally:
        del os.environ["PIPEMAX_ATTN_CHUNK_PAGES"]
    st = runner.stage
    st.prefetch_kv(0)
    outs = [torch.empty_like(hin) for _ in range(40)]
    for hout in outs:
        st.decode_step(0, hin.data_ptr(), hout.data_ptr(), cur)
    st.sync()
    for r, o in enumerate(outs):
        np.testing.assert_array_equal(o.cpu().view(torch.int16).numpy(), a[r], err_msg=f"step {r} differs between two runs")
    assert np.isfinite(np.stack([x.view(np.uint16).astype(np.uint32) << 16 for x in a]).view(np.float32)).all()
    st.destroy()
