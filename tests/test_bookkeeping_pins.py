"""Pins of the bookkeeping oracle: Eq. 3, Eq. 1 / App. A.2, KV sizing (CPU only)."""
import os

import pytest

from oracle import bookkeeping_oracle as bk

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _kv(path):
    out = {}
    for line in open(os.path.join(GOLD, path)):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


@pytest.mark.parametrize("n", [2, 3, 4, 6, 8])
def test_cyclic_roles_eq3(n):
    for t in range(5 * n):
        i, j, k = bk.cyclic_roles(t, n)
        assert i == t % n
        assert j == bk.cyclic_roles(t + 1, n)[0]          # prefetched now = executed next
        assert k == bk.cyclic_roles(t - 1 + n, n)[0]      # overwritten now = executed last
        assert 0 <= i < n and 0 <= j < n and 0 <= k < n
        if n >= 3:
            assert len({i, j, k}) == 3
    # every batch executes exactly once per cycle
    assert sorted(bk.cyclic_roles(t, n)[0] for t in range(n)) == list(range(n))
    # the literal example of Eq. 3 for n = 4, t = 5
    if n == 4:
        assert bk.cyclic_roles(5, 4) == (1, 2, 0)
        assert bk.cyclic_roles(4, 4) == (0, 1, 3)


def test_kv_footprint_example_of_the_paper():
    g = _kv("kv_footprint_example.txt")
    per_tok = bk.kv_bytes_per_token(int(g["layers"]), int(g["kv_heads"]), int(g["head_dim"]),
                                    int(g["elem_bytes"]))
    assert per_tok == 262144
    total_gb = per_tok * g["batch"] * g["seq_len"] / 1e9
    assert abs(total_gb - g["paper_gb"]) / g["paper_gb"] < 0.04     # 137.4 GB vs "about 133 GB"


def test_kv_bytes_per_token_of_the_benchmark_stages():
    from paper_2605_02189_amd.synth_inputs import CONFIGS
    expect = {"C1": 2 * 1024, "C2": 32 * 1024, "C3": 32 * 1024, "C4": 40 * 1024, "C5": 40 * 1024}
    for name, shp in CONFIGS.items():
        assert bk.kv_bytes_per_token(shp.n_layers, shp.n_kv_heads, shp.head_dim, shp.elem_bytes) \
            == expect[name] == shp.kv_bytes_per_token
        assert shp.page_bytes == 16 * expect[name]


def test_token_budget_eq1_and_appendix_a2():
    M, W, T = 32e9, 140e9, 327680.0
    for n in (4, 8):
        cap = bk.system_token_capacity(M, W, n, T)
        assert cap == pytest.approx((M - W / n) / (T / n))          # M_kv / T_gpu
        assert bk.token_budget_per_batch(M, W, n, T) == pytest.approx(cap / n)
    # more pipeline stages raise the per-batch budget only through the W/n term
    assert bk.token_budget_per_batch(M, W, 8, T) > bk.token_budget_per_batch(M, W, 4, T)
    assert bk.token_budget_per_batch(M, 0.0, 4, T) == pytest.approx(M / T)


def test_synthetic_lengths_bracket_table2():
    from paper_2605_02189_amd.synth_inputs import CONFIGS
    g = _kv("table2_lengths.txt")
    share = g["sharegpt_in_avg"] + g["sharegpt_out_avg"]
    longb = g["longbench_in_avg"] + g["longbench_out_avg"]
    assert share < CONFIGS["C2"].ctx_lo + CONFIGS["C2"].decode_steps        # C2 sits above ShareGPT's mean
    assert CONFIGS["C3"].ctx_lo <= share <= CONFIGS["C3"].ctx_hi
    assert CONFIGS["C3"].ctx_lo <= longb <= CONFIGS["C3"].ctx_hi


def test_residency_model_cycle_with_two_arenas():
    """Config-1 schedule: 4 micro-batches, GPU pool of two micro-batches' pages."""
    n, b, L, pt = 4, 8, 128, 16
    per_mb = b * (L // pt + 1)
    m = bk.ResidencyModel(n, pt, max_ctx=L + 16, gpu_pages=2 * per_mb, host_pages=n * per_mb)
    for mb in range(n):
        m.mb_define(mb, [L] * b)
    m.prefetch(0)
    for t in range(16):
        i, j, k = bk.cyclic_roles(t, n)
        if t > 0:
            m.evict(k)
        m.prefetch(j)
        m.decode_step(i)
        on_gpu = [mb for mb in range(n) if m.resident(mb, 0)]
        assert sorted(on_gpu) == sorted({i, j})                   # 2 of 4 on the GPU side
        assert sum(1 for mb in range(n) if not m.resident(mb, 0)) == 2
    assert [m.ctx_lens(mb)[0] for mb in range(n)] == [L + 4] * n
    assert m.n_pages(0, 0) == 9


def test_residency_model_errors():
    m = bk.ResidencyModel(2, 16, max_ctx=40, gpu_pages=3, host_pages=10)
    m.mb_define(0, [16, 17])            # 1 + 2 host pages
    m.mb_define(1, [40])                # 3 host pages
    with pytest.raises(bk.BookkeepingError, match="NOT_RESIDENT"):
        m.decode_step(0)
    m.prefetch(0)                       # takes all 3 GPU pages
    with pytest.raises(bk.BookkeepingError, match="POOL_EXHAUSTED"):
        m.prefetch(1)
    with pytest.raises(bk.BookkeepingError, match="POOL_EXHAUSTED"):
        m.decode_step(0)                # seq 0 is at a page boundary and needs a 4th GPU page
    m.evict(0, [1])
    m.prefetch(0, [1])
    m.evict(0)
    m.prefetch(1)
    with pytest.raises(bk.BookkeepingError, match="STATE"):
        m.decode_step(1)                # already at max_ctx
    with pytest.raises(bk.BookkeepingError, match="ARG"):
        m.mb_define(1, [1])


def test_residency_model_host_reservation():
    m = bk.ResidencyModel(1, 16, max_ctx=64, gpu_pages=10, host_pages=10, host_reserve_tokens=20)
    m.mb_define(0, [16, 60])            # holds pages for 36 -> 3 and min(64, 80) -> 4
    assert m.host_free == 3
    m.prefetch(0)                       # 1 + 4 GPU pages
    assert m.gpu_free == 5
    for _ in range(4):
        m.decode_step(0)                # 16 -> 17 takes a GPU page and a reserved host page
    assert m.gpu_free == 4 and m.host_free == 3
    assert m.ctx_lens(0) == [20, 64]
    with pytest.raises(bk.BookkeepingError, match="STATE"):
        m.decode_step(0)
