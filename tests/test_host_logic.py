"""CPU-only tests of the C-ABI library: it loads, exports what the header declares, and its
host-side planning code (page allocator, copy-run planner, in-page layout) behaves."""
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_symbol_of_the_header(lib):
    hdr = open(os.path.join(ROOT, "include", "pipemax.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(pipemax_[a-z_]+)\s*\(", hdr))
    assert declared == set(lib.SYMBOLS)
    for name in declared:
        assert getattr(lib._lib, name) is not None
    assert "gfx950" in lib.version()


def test_struct_sizes_match_the_header(lib):
    import ctypes as C
    # pipemax_config_t: 6 int32, 2 float, 5 int32, (pad) 2 uint64, int32, uint32, 2 int32
    assert C.sizeof(lib.Config) == 88
    assert lib.Config.gpu_kv_bytes.offset == 56
    assert C.sizeof(lib.Stats) == 8 * 8 + 4 * 8 + lib.N_KCLASS * 16 + 5 * 4 + 4 + 8 + 8 + 8


def test_stage_create_fails_loudly_without_a_gpu_or_with_bad_shapes(lib):
    kw = dict(n_layers=1, hidden=64, n_q_heads=2, n_kv_heads=1, head_dim=32, ffn=64, rope_base=1e4,
              rms_eps=1e-5, dtype=lib.F32, n_microbatches=1, max_seqs_per_mb=1, max_ctx=32,
              gpu_kv_bytes=1 << 20, host_kv_bytes=1 << 20)
    for bad in (dict(page_tokens=8), dict(head_dim=48), dict(n_q_heads=3, n_kv_heads=2), dict(dtype=7),
                dict(n_layers=0)):
        with pytest.raises(lib.PipemaxError) as e:
            lib.Stage(**{**kw, **bad})
        assert e.value.code == lib.ERR_ARG
    import torch
    if not torch.cuda.is_available():
        with pytest.raises(lib.PipemaxError) as e:
            lib.Stage(**kw)
        assert e.value.code == lib.ERR_HIP


def test_pool_is_lowest_index_first_and_all_or_nothing(lib):
    p = lib.Pool(10)
    assert list(p.alloc(4)) == [0, 1, 2, 3]
    assert list(p.alloc(2)) == [4, 5]
    p.free([1, 2, 5])
    assert p.free_count() == 7
    assert list(p.alloc(4)) == [1, 2, 5, 6]                      # lowest free indices, across intervals
    with pytest.raises(lib.PipemaxError) as e:
        p.alloc(4)                                               # only 3 left
    assert e.value.code == lib.ERR_POOL_EXHAUSTED
    assert p.free_count() == 3                                   # nothing taken
    assert list(p.alloc(3)) == [7, 8, 9]
    for bad in ([0, 0], [10], [-1]):
        with pytest.raises(lib.PipemaxError):
            p.free(bad)
    p.free([0])
    with pytest.raises(lib.PipemaxError):
        p.free([0])                                              # double free
    assert p.free_count() == 1


def test_pool_random_against_a_set_model(lib):
    rng = np.random.default_rng(0)
    n = 257
    p = lib.Pool(n)
    free, held = set(range(n)), []
    for _ in range(400):
        if held and rng.random() < 0.45:
            k = int(rng.integers(1, len(held) + 1))
            idx = rng.choice(len(held), size=k, replace=False)
            pages = [held[i] for i in idx]
            held = [h for i, h in enumerate(held) if i not in set(idx.tolist())]
            p.free(pages)
            free |= set(pages)
        else:
            k = int(rng.integers(0, 40))
            if k > len(free):
                with pytest.raises(lib.PipemaxError):
                    p.alloc(k)
                continue
            got = list(p.alloc(k))
            assert got == sorted(free)[:k]
            free -= set(got)
            held += got
        assert p.free_count() == len(free)


def test_copy_runs_merge_consecutive_pairs_only(lib):
    runs = lib.plan_copy_runs([0, 1, 2, 5, 6, 9], [10, 11, 12, 13, 14, 20], 128)
    assert runs.tolist() == [[0, 10, 3], [5, 13, 2], [9, 20, 1]]
    runs = lib.plan_copy_runs(np.arange(10), np.arange(10) + 100, 4)
    assert runs.tolist() == [[0, 100, 4], [4, 104, 4], [8, 108, 2]]
    runs = lib.plan_copy_runs([3, 4, 5], [7, 9, 10], 128)           # dst not consecutive at first pair
    assert runs.tolist() == [[3, 7, 1], [4, 9, 2]]
    assert lib.plan_copy_runs([], [], 8).shape == (0, 3)
    # the runs cover every pair exactly once, in order
    rng = np.random.default_rng(1)
    src = np.sort(rng.choice(1000, 300, replace=False))
    dst = np.sort(rng.choice(1000, 300, replace=False))
    runs = lib.plan_copy_runs(src, dst, 16)
    s = np.concatenate([np.arange(a, a + c) for a, _, c in runs])
    d = np.concatenate([np.arange(b, b + c) for _, b, c in runs])
    np.testing.assert_array_equal(s, src)
    np.testing.assert_array_equal(d, dst)
    assert runs[:, 2].max() <= 16


@pytest.mark.parametrize("d", [32, 64, 128])
def test_page_layout_is_a_bijection_with_the_documented_order(lib, d):
    nl, hkv = 3, 2
    total = nl * hkv * 2 * 16 * d
    seen = np.zeros(total, dtype=np.int32)
    for layer in range(nl):
        for head in range(hkv):
            for kv in range(2):
                base = ((layer * hkv + head) * 2 + kv) * 16 * d        # [layer][head][K|V] sub-blocks
                for tok in range(16):
                    for dd in range(d):
                        off = lib.page_elem_offset(nl, hkv, d, layer, kv, head, tok, dd)
                        if kv == 0:
                            want = base + ((dd // 8) * 16 + tok) * 8 + dd % 8
                        else:
                            want = base + ((((dd // 32) * 4 + tok // 4) * 16 + dd % 16) * 2 + (dd // 16) % 2) * 4 + tok % 4
                        assert off == want
                        seen[off] += 1
    assert np.all(seen == 1)
    assert lib.page_elem_offset(nl, hkv, d, nl, 0, 0, 0, 0) == -1
    assert lib.page_elem_offset(nl, hkv, d, 0, 0, 0, 16, 0) == -1
    assert lib.page_elem_offset(nl, hkv, 48, 0, 0, 0, 0, 0) == -1


def test_gemm_split_plan_and_launch_geometry_agree(lib):
    """The consumers of the split-K partials sum `planned` slices while the GEMM's grid has `launched` splits: the
    two must be the same number for every shape, the splits must cover K, and k ranges come in pairs of k-steps
    (the ring kernel's slots) whenever K allows it."""
    for rows in (129, 150, 256, 257, 512, 600, 768, 1024):
        for n_cols in (256, 1024, 4096, 6144, 10240, 28672, 57344):
            for k in (512, 1024, 2816, 4096, 8192, 14336, 16384, 28672, 4112):
                planned, launched, ksp = lib.plan_gemm_splits(rows, n_cols, k)
                kt = k // 16
                assert planned == launched >= 1, (rows, n_cols, k)
                assert ksp * launched >= kt > ksp * (launched - 1), (rows, n_cols, k)
                assert launched <= max(1, kt // 16)
                if kt % 2 == 0 and launched > 1:
                    assert ksp % 2 == 0, (rows, n_cols, k)
    # 96 column-row blocks (the 8B stage's QKV matrix at 1024 rows): three splits would be 288 work-groups, i.e.
    # two rounds on 256 compute units; the plan takes two
    assert lib.plan_gemm_splits(1024, 6144, 4096)[0] == 2
    # a matrix with more blocks than compute units is not split at all
    assert lib.plan_gemm_splits(1024, 28672, 4096)[0] == 1
    # a single row block streams every weight tile once: its splits leave an eighth of the 256 compute units free
    # (the 70B-sized stage's 256-row GEMMs), while several row blocks, which share tiles, may fill the chip
    for n_cols, k in ((8192, 8192), (8192, 28672), (10240, 8192)):
        splits = lib.plan_gemm_splits(256, n_cols, k)[0]
        assert 1 < splits and (n_cols // 256) * splits <= 224, (n_cols, k, splits)
    assert lib.plan_gemm_splits(1024, 4096, 4096)[0] * 4 * (4096 // 256) == 256
    with pytest.raises(lib.PipemaxError):
        lib.plan_gemm_splits(256, 300, 4096)


def test_attention_chunk_plan_covers_the_context_with_even_chunks(lib):
    """The decode attention's chunking: every plan covers the longest context (chunks x pages per chunk >= its
    pages), a work-group never gets more than 256 pages, chunks are even (no chunk is more than one page short of
    the others), and the cases the benchmark configurations hit come out as measured best: one chunk for 256
    sequences of 2049 tokens, two halves (129 + 128 pages) for 4097 tokens -- not a full work-group and a
    one-page rest."""
    def pages(tokens):
        return -(-tokens // 16)
    for n_seqs, hkv, tokens in ((256, 8, 2049), (256, 8, 4097), (64, 8, 1025), (1, 1, 1), (1, 8, 40000), (3, 1, 3000),
                                (128, 8, 4100), (256, 8, 4096), (2, 2, 4113), (7, 4, 257 * 16), (5, 8, 8193)):
        total = n_seqs * pages(tokens)
        cp, nch, per_wave = lib.plan_attention_chunks(n_seqs, hkv, tokens, total)
        npg = pages(tokens)
        assert per_wave == (n_seqs * hkv >= 2 * 256)
        assert 8 <= cp and (per_wave or cp <= 256) and nch >= 1, (n_seqs, hkv, tokens, cp, nch)
        assert cp * nch >= npg, (n_seqs, hkv, tokens, cp, nch)
        assert nch == -(-npg // cp)
        last = npg - (nch - 1) * cp                     # pages of the last chunk
        assert last >= 1 and (cp - last <= nch or cp == 8), (n_seqs, hkv, tokens, cp, nch, last)
    # uniform batches with enough (sequence, head) pairs: a wave per pair, the whole context in one chunk
    assert lib.plan_attention_chunks(256, 8, 2049, 256 * 129) == (129, 1, True)
    assert lib.plan_attention_chunks(256, 8, 4097, 256 * 257) == (257, 1, True)
    # on a chip with more compute units the same step goes to work-groups of four waves, at most 256 pages each
    assert lib.plan_attention_chunks(256, 8, 2049, 256 * 129, 2048) == (129, 1, False)
    assert lib.plan_attention_chunks(256, 8, 4097, 256 * 257, 2048) == (129, 2, False)
    assert lib.plan_attention_chunks(64, 8, 1025, 64 * 65) == (33, 2, True)        # few pairs: two waves per pair
    assert lib.plan_attention_chunks(32, 8, 1025, 32 * 65) == (65, 1, False)
    # a ragged batch whose longest sequence would outlast everything else is cut into several chunks
    cp, nch, _ = lib.plan_attention_chunks(3, 1, 3000, pages(3000) + pages(41) + pages(1026))
    assert nch > 1
    cp, nch, per_wave = lib.plan_attention_chunks(128, 8, 4097, 127 * pages(1600) + 257)
    assert per_wave and nch > 1 and cp * nch >= 257
    import pytest
    with pytest.raises(lib.PipemaxError):
        lib.plan_attention_chunks(0, 8, 100, 7)
