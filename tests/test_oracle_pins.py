"""Pins of the CPU oracle against things other than itself (CPU only).

Each test fixes the oracle to a closed form, an invariant, a brute-force
definition written independently in this file, or a library routine.
"""
import cmath
import math

import numpy as np
import pytest

from oracle import stage_oracle as so

from conftest import rel_l2


# --------------------------------------------------------------------------
# an independent brute-force decoder slice: scalar loops, float64, complex RoPE,
# full causal recompute over the whole prefix (no cache anywhere)
# --------------------------------------------------------------------------
def _bf_matvec(x, W):                      # y[n] = sum_k x[k] W[k][n]
    K, N = len(W), len(W[0])
    return [sum(x[k] * W[k][n] for k in range(K)) for n in range(N)]


def _bf_rms(x, g, eps):
    ms = sum(v * v for v in x) / len(x)
    r = 1.0 / math.sqrt(ms + eps)
    return [v * r * gg for v, gg in zip(x, g)]


def _bf_rope(head, pos, base):
    d = len(head)
    out = [0.0] * d
    for j in range(d // 2):
        z = complex(head[j], head[j + d // 2]) * cmath.exp(1j * pos * base ** (-2.0 * j / d))
        out[j], out[j + d // 2] = z.real, z.imag
    return out


def brute_force_last_token(W, xs, Hq, Hkv, d, F, base, eps):
    """xs: list over positions 0..t of the stage's input vector for that position.
    Returns the stage output for the last position, recomputing every position."""
    G = Hq // Hkv
    T = len(xs)
    cur = [list(map(float, x)) for x in xs]            # residual stream of every position
    for L in W:
        wqkv, wo, wgu, wd, g1, g2 = L
        qs, ks, vs = [], [], []
        for p in range(T):
            xn = _bf_rms(cur[p], g1, eps)
            qkv = _bf_matvec(xn, wqkv)
            q = [qkv[u * d:(u + 1) * d] for u in range(Hq)]
            k = [qkv[Hq * d + c * d: Hq * d + (c + 1) * d] for c in range(Hkv)]
            v = [qkv[(Hq + Hkv) * d + c * d: (Hq + Hkv) * d + (c + 1) * d] for c in range(Hkv)]
            qs.append([_bf_rope(h_, p, base) for h_ in q])
            ks.append([_bf_rope(h_, p, base) for h_ in k])
            vs.append(v)
        nxt = []
        for p in range(T):
            o = []
            for u in range(Hq):
                c = u // G
                sc = [sum(qs[p][u][e] * ks[t][c][e] for e in range(d)) / math.sqrt(d)
                      for t in range(p + 1)]                       # causal: t <= p
                m = max(sc)
                ex = [math.exp(s - m) for s in sc]
                z = sum(ex)
                o += [sum(ex[t] / z * vs[t][c][e] for t in range(p + 1)) for e in range(d)]
            x1 = [a + b for a, b in zip(cur[p], _bf_matvec(o, wo))]
            xn2 = _bf_rms(x1, g2, eps)
            gu = _bf_matvec(xn2, wgu)
            act = [(gu[f] / (1.0 + math.exp(-gu[f]))) * gu[F + f] for f in range(F)]
            nxt.append([a + b for a, b in zip(x1, _bf_matvec(act, wd))])
        cur = nxt
    return cur[-1]


def _tiny_weights(rng, nl, h, Hq, Hkv, d, F, scale=0.3):
    Ws = []
    for _ in range(nl):
        Ws.append((rng.normal(0, scale, (h, (Hq + 2 * Hkv) * d)),
                   rng.normal(0, scale, (Hq * d, h)),
                   rng.normal(0, scale, (h, 2 * F)),
                   rng.normal(0, scale, (F, h)),
                   1.0 + 0.2 * rng.normal(size=h),
                   1.0 + 0.2 * rng.normal(size=h)))
    return Ws


@pytest.mark.parametrize("dtype,tol", [(np.float64, 1e-11), (np.float32, 1e-5)])
def test_incremental_decode_equals_full_prefix_recompute(dtype, tol):
    """Decode with cached K,V must equal recomputing the whole prefix (Sec. 2.1)."""
    rng = np.random.default_rng(7)
    nl, h, Hq, Hkv, d, F, base, eps = 2, 12, 4, 2, 6, 10, 100.0, 1e-5
    W = _tiny_weights(rng, nl, h, Hq, Hkv, d, F)
    orc = so.StageOracle(nl, h, Hq, Hkv, d, F, base, eps, dtype=dtype)
    for l, w in enumerate(W):
        orc.set_layer_weights(l, *w)
    b, T = 2, 5
    empty = [np.zeros((0, Hkv, d))] * nl
    for s in range(b):
        orc.define_sequence(0, s, empty, empty)
    xs = rng.normal(size=(T, b, h))
    for t in range(T):
        out, per_layer = orc.decode_step(0, xs[t])
        assert per_layer.shape == (nl, b, h)
        np.testing.assert_array_equal(per_layer[-1], out)
        for s in range(b):
            ref = brute_force_last_token([tuple(a.tolist() for a in w) for w in W],
                                         [xs[u, s].tolist() for u in range(t + 1)],
                                         Hq, Hkv, d, F, base, eps)
            assert rel_l2(out[s], ref) < tol, (t, s)
            assert orc.ctx_len(0, s) == t + 1


def test_prefix_cache_given_equals_cache_built_by_decoding():
    """Starting from a supplied prefix cache == having decoded those tokens."""
    rng = np.random.default_rng(3)
    nl, h, Hq, Hkv, d, F = 2, 16, 4, 2, 8, 12
    W = _tiny_weights(rng, nl, h, Hq, Hkv, d, F)
    A = so.StageOracle(nl, h, Hq, Hkv, d, F, 10000.0, 1e-5, dtype=np.float64)
    B = so.StageOracle(nl, h, Hq, Hkv, d, F, 10000.0, 1e-5, dtype=np.float64)
    for l, w in enumerate(W):
        A.set_layer_weights(l, *w)
        B.set_layer_weights(l, *w)
    empty = [np.zeros((0, Hkv, d))] * nl
    A.define_sequence(0, 0, empty, empty)
    xs = rng.normal(size=(4, 1, h))
    for t in range(3):
        A.decode_step(0, xs[t])
    B.define_sequence(0, 0, [A.cached_kv(0, 0, l)[0].copy() for l in range(nl)],
                      [A.cached_kv(0, 0, l)[1].copy() for l in range(nl)])
    oa, _ = A.decode_step(0, xs[3])
    ob, _ = B.decode_step(0, xs[3])
    np.testing.assert_array_equal(oa, ob)


def test_rows_of_a_microbatch_are_independent():
    rng = np.random.default_rng(11)
    nl, h, Hq, Hkv, d, F = 2, 16, 4, 2, 8, 12
    W = _tiny_weights(rng, nl, h, Hq, Hkv, d, F)
    full = so.StageOracle(nl, h, Hq, Hkv, d, F, 10000.0, 1e-5, dtype=np.float64)
    one = so.StageOracle(nl, h, Hq, Hkv, d, F, 10000.0, 1e-5, dtype=np.float64)
    for l, w in enumerate(W):
        full.set_layer_weights(l, *w)
        one.set_layer_weights(l, *w)
    b = 3
    lens = [5, 1, 9]
    caches = [[(rng.normal(size=(L, Hkv, d)), rng.normal(size=(L, Hkv, d))) for _ in range(nl)]
              for L in lens]
    for s in range(b):
        full.define_sequence(0, s, [c[0] for c in caches[s]], [c[1] for c in caches[s]])
    one.define_sequence(0, 2, [c[0] for c in caches[2]], [c[1] for c in caches[2]])
    x = rng.normal(size=(b, h))
    of, _ = full.decode_step(0, x)
    oo, _ = one.decode_step(0, x[2:3], seqs=[2])
    np.testing.assert_allclose(oo[0], of[2], rtol=1e-12, atol=1e-12)


# --------------------------------------------------------------------------
# attention
# --------------------------------------------------------------------------
def test_softmax_rows_sum_to_one():
    rng = np.random.default_rng(0)
    for dt, tol in ((np.float32, 1e-6), (np.float64, 1e-14)):
        q = rng.normal(size=(8, 16)).astype(dt) * 3
        K = rng.normal(size=(37, 2, 16)).astype(dt)
        V = rng.normal(size=(37, 2, 16)).astype(dt)
        _, w = so.attention_decode(q, K, V, return_weights=True)
        assert w.shape == (8, 37)
        assert np.all(w >= 0)
        assert np.max(np.abs(w.sum(axis=1) - 1.0)) < tol


def test_attention_over_one_cached_token_returns_its_v_exactly():
    rng = np.random.default_rng(1)
    Hq, Hkv, d = 6, 3, 8
    q = rng.normal(size=(Hq, d)).astype(np.float32)
    K = rng.normal(size=(1, Hkv, d)).astype(np.float32)
    V = rng.normal(size=(1, Hkv, d)).astype(np.float32)
    o = so.attention_decode(q, K, V)
    for u in range(Hq):
        np.testing.assert_array_equal(o[u], V[0, u // (Hq // Hkv)])     # bit for bit


def test_equal_scores_give_mean_of_v():
    rng = np.random.default_rng(2)
    q = np.zeros((4, 8))
    K = rng.normal(size=(13, 2, 8))
    V = rng.normal(size=(13, 2, 8))
    o = so.attention_decode(q, K, V)
    for u in range(4):
        np.testing.assert_allclose(o[u], V[:, u // 2].mean(axis=0), rtol=1e-13, atol=1e-13)


def test_attention_prefers_the_matching_key():
    """Sign and scale of the score: a key equal to a large multiple of q wins."""
    d = 16
    q = np.ones((1, d))
    K = np.zeros((3, 1, d))
    K[1, 0] = 50.0
    K[2, 0] = -50.0
    V = np.arange(3, dtype=np.float64).reshape(3, 1, 1) * np.ones((3, 1, d))
    o, w = so.attention_decode(q, K, V, return_weights=True)
    assert w[0, 1] > 0.999999 and w[0, 2] < 1e-12
    # exact value of the scale: scores are q.k / sqrt(d) = (0, 200, -200)
    ref = np.exp(np.array([0.0, 50.0 * d / math.sqrt(d), -50.0 * d / math.sqrt(d)]) - 50.0 * d / math.sqrt(d))
    np.testing.assert_allclose(w[0], ref / ref.sum(), rtol=1e-12)


def test_gqa_equals_mha_with_duplicated_kv_heads():
    rng = np.random.default_rng(4)
    Hq, Hkv, d, T = 8, 2, 8, 21
    G = Hq // Hkv
    q = rng.normal(size=(Hq, d))
    K = rng.normal(size=(T, Hkv, d))
    V = rng.normal(size=(T, Hkv, d))
    o_gqa = so.attention_decode(q, K, V)
    o_mha = so.attention_decode(q, np.repeat(K, G, axis=1), np.repeat(V, G, axis=1))
    np.testing.assert_array_equal(o_gqa, o_mha)


def test_attention_against_torch_cpu_library_ops():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    Hq, Hkv, d, T = 8, 4, 32, 77
    q = rng.normal(size=(Hq, d))
    K = rng.normal(size=(T, Hkv, d))
    V = rng.normal(size=(T, Hkv, d))
    tq = torch.from_numpy(q)
    tK = torch.from_numpy(K).repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)   # [Hq, T, d]
    tV = torch.from_numpy(V).repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(
        tq[:, None, :], tK, tV)[:, 0, :].numpy()
    np.testing.assert_allclose(so.attention_decode(q, K, V), ref, rtol=1e-11, atol=1e-12)
    o32 = so.attention_decode(q.astype(np.float32), K.astype(np.float32), V.astype(np.float32))
    assert rel_l2(o32, ref) < 1e-6


# --------------------------------------------------------------------------
# RoPE
# --------------------------------------------------------------------------
def test_rope_position_zero_is_identity_and_pairs_keep_their_norm():
    rng = np.random.default_rng(6)
    v = rng.normal(size=(3, 5, 16))
    np.testing.assert_array_equal(so.rope(v, np.zeros(3), 10000.0), v)
    r = so.rope(v, np.array([1, 17, 4000]), 10000.0)
    n0 = v[..., :8] ** 2 + v[..., 8:] ** 2
    n1 = r[..., :8] ** 2 + r[..., 8:] ** 2
    np.testing.assert_allclose(n1, n0, rtol=1e-12)


def test_rope_inner_product_depends_only_on_relative_position():
    rng = np.random.default_rng(8)
    q = rng.normal(size=(1, 32))
    k = rng.normal(size=(1, 32))
    def ip(m, n):
        return float(np.sum(so.rope(q, m, 500000.0) * so.rope(k, n, 500000.0)))
    for (m, n), (m2, n2) in [((5, 2), (103, 100)), ((40, 40), (0, 0)), ((7, 19), (1007, 1019))]:
        assert abs(ip(m, n) - ip(m2, n2)) < 1e-10


def test_rope_closed_form_small_case():
    """d = 4, base = 100: theta = (1, 0.1); pairs are (0, 2) and (1, 3); rotation is
    counter-clockwise by pos*theta (x' = x cos - y sin, y' = y cos + x sin)."""
    v = np.array([[1.0, 0.0, 0.0, 1.0]])
    r = so.rope(v, 2, 100.0)[0]
    np.testing.assert_allclose(r, [math.cos(2.0), -math.sin(0.2), math.sin(2.0), math.cos(0.2)],
                               rtol=1e-14, atol=1e-15)


def test_rope_fp32_uses_angles_rounded_once():
    v = np.ones((1, 64), dtype=np.float32)
    r32 = so.rope(v, 4095, 500000.0)
    r64 = so.rope(v.astype(np.float64), 4095, 500000.0)
    assert np.max(np.abs(r32 - r64)) < 3e-7


# --------------------------------------------------------------------------
# RMSNorm, SiLU
# --------------------------------------------------------------------------
def test_rmsnorm_unit_gain_gives_unit_rms_and_is_scale_invariant():
    rng = np.random.default_rng(9)
    x = rng.normal(size=(5, 64)) * 7
    g = np.ones(64)
    y = so.rmsnorm(x, g, 0.0)
    np.testing.assert_allclose(np.sqrt(np.mean(y * y, axis=-1)), 1.0, rtol=1e-13)
    np.testing.assert_allclose(so.rmsnorm(3.5 * x, g, 0.0), y, rtol=1e-13)
    # eps enters inside the square root, added to the mean square
    x1 = np.full((1, 4), 2.0)
    np.testing.assert_allclose(so.rmsnorm(x1, np.array([1.0, 2.0, 3.0, 4.0]), 5.0),
                               [[2 / 3.0, 4 / 3.0, 2.0, 8 / 3.0]], rtol=1e-14)


def test_silu_closed_forms():
    z = np.linspace(-30, 30, 241)
    np.testing.assert_allclose(so.silu(z) - so.silu(-z), z, atol=1e-12)
    assert so.silu(np.array([0.0]))[0] == 0.0
    assert abs(so.silu(np.array([40.0]))[0] - 40.0) < 1e-12
    assert abs(so.silu(np.array([-40.0]))[0]) < 1e-12
    np.testing.assert_allclose(so.silu(np.array([1.0]))[0], 1.0 / (1.0 + math.exp(-1.0)), rtol=1e-15)


# --------------------------------------------------------------------------
# the layer: branch structure and weight orientation
# --------------------------------------------------------------------------
def test_zero_output_projections_make_the_layer_the_identity():
    rng = np.random.default_rng(10)
    nl, h, Hq, Hkv, d, F = 1, 16, 4, 2, 8, 12
    w = list(_tiny_weights(rng, nl, h, Hq, Hkv, d, F)[0])
    w[1] = np.zeros_like(w[1])
    w[3] = np.zeros_like(w[3])
    orc = so.StageOracle(nl, h, Hq, Hkv, d, F, 10000.0, 1e-5, dtype=np.float64)
    orc.set_layer_weights(0, *w)
    orc.define_sequence(0, 0, [rng.normal(size=(3, Hkv, d))], [rng.normal(size=(3, Hkv, d))])
    x = rng.normal(size=(1, h))
    out, _ = orc.decode_step(0, x)
    np.testing.assert_array_equal(out, x)
    assert orc.ctx_len(0, 0) == 4


def test_appended_kv_is_the_projected_and_rotated_new_token():
    """K row = rope(rmsnorm(x) @ Wk, pos = L), V row = rmsnorm(x) @ Wv (no rotation)."""
    rng = np.random.default_rng(12)
    nl, h, Hq, Hkv, d, F = 1, 8, 2, 1, 4, 6
    w = _tiny_weights(rng, nl, h, Hq, Hkv, d, F)[0]
    orc = so.StageOracle(nl, h, Hq, Hkv, d, F, 100.0, 1e-5, dtype=np.float64)
    orc.set_layer_weights(0, *w)
    L = 3
    orc.define_sequence(0, 0, [rng.normal(size=(L, Hkv, d))], [rng.normal(size=(L, Hkv, d))])
    x = rng.normal(size=(1, h))
    orc.decode_step(0, x)
    Kc, Vc = orc.cached_kv(0, 0, 0)
    xn = _bf_rms(x[0].tolist(), w[4].tolist(), 1e-5)
    qkv = _bf_matvec(xn, w[0].tolist())
    k_ref = _bf_rope(qkv[Hq * d: Hq * d + d], L, 100.0)
    v_ref = qkv[(Hq + Hkv) * d:]
    np.testing.assert_allclose(Kc[L, 0], k_ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(Vc[L, 0], v_ref, rtol=1e-12, atol=1e-13)


def test_fp32_oracle_agrees_with_fp64_oracle_on_config1_shapes():
    from paper_2605_02189_amd.synth_inputs import CONFIGS, SynthInputs
    shp = CONFIGS["C1"]
    syn = SynthInputs(shp, seed=1, pool_elems=1 << 21, gain_jitter=0.1)
    outs = {}
    for dt in (np.float32, np.float64):
        orc = so.StageOracle(shp.n_layers, shp.hidden, shp.n_q_heads, shp.n_kv_heads, shp.head_dim,
                             shp.ffn, shp.rope_base, shp.rms_eps, dtype=dt)
        for l in range(shp.n_layers):
            orc.set_layer_weights(l, **{k: syn.as_f32(v) for k, v in syn.weights(l).items()})
        L = int(syn.ctx_lens(0)[0])
        for s in range(2):
            kv = [syn.kv_prefix(0, s, l, L) for l in range(shp.n_layers)]
            orc.define_sequence(0, s, [k for k, _ in kv], [v for _, v in kv])
        x = syn.as_f32(syn.hidden(0, 2))
        for _ in range(3):
            out, per_layer = orc.decode_step(0, x)
        outs[dt] = per_layer
    for l in range(shp.n_layers):
        assert rel_l2(outs[np.float32][l], outs[np.float64][l]) < 2e-6


def test_widen_bf16_is_exact():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x7F80], dtype=np.uint16)
    np.testing.assert_array_equal(so.widen_bf16(bits),
                                  np.array([1.0, -1.0, 3.140625, 0.0, np.inf], dtype=np.float32))


def test_operand_round_mode_is_the_plain_oracle_plus_a_small_perturbation():
    """The diagnostic operand-rounding mode: an identity hook leaves every bit of the result alone (the hook is
    applied outside the arithmetic), and bf16 rounding moves a one-layer result by the size operand rounding has
    (between 2e-4 and 1e-2), never by more."""
    rng = np.random.default_rng(5)
    nl, h, Hq, Hkv, d, F = 2, 32, 4, 2, 8, 48
    Ws = _tiny_weights(rng, nl, h, Hq, Hkv, d, F)
    Kp = [rng.normal(size=(5, Hkv, d)).astype(np.float32) for _ in range(nl)]
    Vp = [rng.normal(size=(5, Hkv, d)).astype(np.float32) for _ in range(nl)]
    x = rng.normal(size=(3, h)).astype(np.float32)

    def bf16(a):
        u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
        r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)) << np.uint32(16)
        return r.view(np.float32).reshape(np.shape(a))

    outs = {}
    for name, hook in (("none", None), ("identity", lambda a: a), ("bf16", bf16)):
        orc = so.StageOracle(nl, h, Hq, Hkv, d, F, 10000.0, 1e-5, operand_round=hook)
        for l, W in enumerate(Ws):
            orc.set_layer_weights(l, *W)
        for s in range(3):
            orc.define_sequence(0, s, Kp, Vp)
        outs[name] = orc.decode_step(0, x)[1]
    np.testing.assert_array_equal(outs["identity"], outs["none"])
    e = rel_l2(outs["bf16"][0], outs["none"][0])
    assert 2e-4 < e < 1e-2, e
