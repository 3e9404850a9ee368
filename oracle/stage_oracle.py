"""Plain CPU oracle of one pipeline stage's decode step (numpy, fp32).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  The product path never calls it and it shares no
code with the HIP kernels.

What it is.  PipeMax (Sec. 3, Sec. 3.3.2 and Sec. 3.4.2) moves the KV cache of
inactive decode batches to host memory and back, and changes the physical page
layout; both change only *where bytes live*.  The paper states that decoding
keeps its autoregressive semantics (Sec. 3.3.2) and that the layout change only
affects storage and transfer (Sec. 3.4.2, block-first layout).  The result of a
stage decode step is therefore the plain definition of a Llama-style decoder
slice run with a KV cache (Sec. 2.1: decode re-uses the cached K,V of the
prefix instead of recomputing them).  This file is that definition written out
with one contiguous K and V array per (micro-batch, sequence, layer): no pages,
no residency, no streams.

The paper inherits the transformer arithmetic from the serving system it builds
on and never spells it out.  The readings taken here (pre-norm residual blocks,
no biases, half-split RoPE pairs, softmax scale 1/sqrt(d), the new token attends
to itself at position L_i) are stated where each function implements them.

Pins (tests/test_oracle_pins.py): incremental-with-cache == brute-force full
causal recompute; softmax rows sum to 1; one cached token returns its V exactly;
uniform scores give the mean of V; GQA reduces to MHA; RoPE identities; RMSNorm
and SiLU closed forms; GEMM against a triple loop; library cross-check of the
attention against torch CPU ops.  Absolute activations are "parity unpinned" by
the paper (it prints none); they are pinned only through those invariants.

Diagnostic mode (not the contract): `operand_round`, when given, is applied where a bf16 matrix-core path has
to store an operand in bf16 (the normalised activations, q after RoPE, the appended K and V, the softmax
weights, the attention output, the SwiGLU output).  With it the oracle emulates what operand rounding alone
costs against the plain fp32 result, which the parity tests use to place their accumulated-error bar; the
default (None) is the plain definition and nothing else compares against the emulation.

Precision: float32 by default (the precision the benchmark spec fixes for the
oracle); every function takes the array dtype it is given, so the pins also run
it in float64 to show that fp32 rounding does not matter at the tolerances used.
RoPE angles are always formed in float64 and rounded once.
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------
# storage helpers (no arithmetic of the method)
# --------------------------------------------------------------------------
def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32, exact."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------
# element-wise pieces
# --------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """y_j = x_j / sqrt(mean_j(x^2) + eps) * g_j over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + x.dtype.type(eps)) * g


def silu(z: np.ndarray) -> np.ndarray:
    """z / (1 + exp(-z))."""
    return z / (1.0 + np.exp(-z))


def rope_angles(pos, d: int, base: float) -> np.ndarray:
    """Angles pos * base^(-2j/d), j in [0, d/2), in float64.  pos: scalar or [b]."""
    j = np.arange(d // 2, dtype=np.float64)
    theta = np.power(np.float64(base), -2.0 * j / np.float64(d))
    return np.multiply.outer(np.asarray(pos, dtype=np.float64), theta)


def rope(v: np.ndarray, pos, base: float) -> np.ndarray:
    """Rotate the pairs (j, j + d/2) of the last axis of v by pos * theta_j.

    v: [..., heads, d] with pos broadcasting over the leading axes
    (pos scalar for [heads, d]; pos [b] for [b, heads, d]).
    """
    d = v.shape[-1]
    half = d // 2
    ang = rope_angles(pos, d, base)                   # [half] or [b, half]
    c = np.cos(ang).astype(v.dtype)
    s = np.sin(ang).astype(v.dtype)
    if ang.ndim == 2:                                 # [b, half] -> [b, 1, half]
        c = c[:, None, :]
        s = s[:, None, :]
    lo, hi = v[..., :half], v[..., half:]
    out = np.empty_like(v)
    out[..., :half] = lo * c - hi * s
    out[..., half:] = hi * c + lo * s
    return out


def softmax_lastaxis(s: np.ndarray) -> np.ndarray:
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention_decode(q: np.ndarray, K: np.ndarray, V: np.ndarray,
                     return_weights: bool = False, weight_round=None):
    """One query token against T cached tokens, grouped-query attention.

    q [Hq, d]; K, V [T, Hkv, d]; query head u reads KV head u // G, G = Hq/Hkv.
    o_u = softmax_t(q_u . K[t, u//G] / sqrt(d)) @ V[:, u//G].   Returns [Hq, d].
    """
    Hq, d = q.shape
    T, Hkv, _ = K.shape
    G = Hq // Hkv
    assert G * Hkv == Hq
    scale = q.dtype.type(1.0 / np.sqrt(np.float64(d)))
    out = np.empty_like(q)
    ws = []
    for u in range(Hq):
        c = u // G
        s = (K[:, c, :] @ q[u]) * scale               # [T]
        w = softmax_lastaxis(s)
        out[u] = (w if weight_round is None else weight_round(w)) @ V[:, c, :]
        if return_weights:
            ws.append(w)
    if return_weights:
        return out, np.stack(ws)
    return out


# --------------------------------------------------------------------------
# the stage
# --------------------------------------------------------------------------
class _Grow:
    """A [T, Hkv, d] array that grows by one token at a time."""

    def __init__(self, init: np.ndarray, dtype):
        init = np.asarray(init, dtype=dtype)
        self.n = init.shape[0]
        cap = max(16, 2 * self.n)
        self.buf = np.zeros((cap,) + init.shape[1:], dtype=dtype)
        self.buf[: self.n] = init

    def append(self, row: np.ndarray) -> None:
        if self.n == self.buf.shape[0]:
            nb = np.zeros((2 * self.n,) + self.buf.shape[1:], dtype=self.buf.dtype)
            nb[: self.n] = self.buf
            self.buf = nb
        self.buf[self.n] = row
        self.n += 1

    @property
    def arr(self) -> np.ndarray:
        return self.buf[: self.n]


class StageOracle:
    """A contiguous slice of decoder layers with per-sequence KV caches.

    Weights are given in the canonical "x @ W" orientation:
      wqkv [h, (Hq+2Hkv)*d]  (columns: all q heads, then all k heads, then all v heads)
      wo   [Hq*d, h]
      wgu  [h, 2F]           (columns: gate, then up)
      wd   [F, h]
      g1, g2 [h]             (RMSNorm gains before attention / before the FFN)
    """

    def __init__(self, n_layers: int, hidden: int, n_q_heads: int, n_kv_heads: int,
                 head_dim: int, ffn: int, rope_base: float, rms_eps: float,
                 dtype=np.float32, operand_round=None):
        self.nl, self.h = n_layers, hidden
        self.Hq, self.Hkv, self.d, self.F = n_q_heads, n_kv_heads, head_dim, ffn
        self.base, self.eps = float(rope_base), float(rms_eps)
        self.dt = np.dtype(dtype)
        self.rnd = operand_round if operand_round is not None else (lambda a: a)
        self.wrnd = operand_round
        self.w = [None] * n_layers
        self.kv = {}          # (mb, seq) -> list over layers of (_Grow K, _Grow V)

    # -- set-up -------------------------------------------------------------
    def set_layer_weights(self, layer, wqkv, wo, wgu, wd, g1, g2):
        f = lambda a: np.ascontiguousarray(a, dtype=self.dt)
        nq, nk = self.Hq * self.d, self.Hkv * self.d
        wqkv = f(wqkv)
        assert wqkv.shape == (self.h, nq + 2 * nk)
        wgu = f(wgu)
        assert wgu.shape == (self.h, 2 * self.F)
        self.w[layer] = dict(
            wq=wqkv[:, :nq], wk=wqkv[:, nq:nq + nk], wv=wqkv[:, nq + nk:],
            wo=f(wo), wg=wgu[:, : self.F], wu=wgu[:, self.F:], wd=f(wd),
            g1=f(g1), g2=f(g2))
        assert self.w[layer]["wo"].shape == (nq, self.h)
        assert self.w[layer]["wd"].shape == (self.F, self.h)

    def define_sequence(self, mb, seq, K_layers, V_layers):
        """K_layers[l], V_layers[l]: [L, Hkv, d] prefix cache of layer l (L may be 0)."""
        assert len(K_layers) == self.nl and len(V_layers) == self.nl
        self.kv[(mb, seq)] = [(_Grow(K_layers[l], self.dt), _Grow(V_layers[l], self.dt))
                              for l in range(self.nl)]

    def ctx_len(self, mb, seq) -> int:
        return self.kv[(mb, seq)][0][0].n

    def cached_kv(self, mb, seq, layer):
        k, v = self.kv[(mb, seq)][layer]
        return k.arr, v.arr

    # -- one decode step ----------------------------------------------------
    def layer_decode(self, layer: int, mb, seqs, x: np.ndarray):
        """x [b, h] -> x_out [b, h] for one layer; appends one token per sequence.

        Returns (x_out, parts) where parts holds the two branch outputs
        (attention branch and FFN branch, each before its residual add).
        """
        W = self.w[layer]
        b = x.shape[0]
        Hq, Hkv, d = self.Hq, self.Hkv, self.d
        xn = self.rnd(rmsnorm(x, W["g1"], self.eps))
        q = (xn @ W["wq"]).reshape(b, Hq, d)
        k = (xn @ W["wk"]).reshape(b, Hkv, d)
        v = (xn @ W["wv"]).reshape(b, Hkv, d)
        pos = np.array([self.kv[(mb, s)][layer][0].n for s in seqs])   # p_i = L_i
        q = self.rnd(rope(q, pos, self.base))
        k = self.rnd(rope(k, pos, self.base))
        v = self.rnd(v)
        o = np.empty((b, Hq, d), dtype=self.dt)
        for r, s in enumerate(seqs):
            Kc, Vc = self.kv[(mb, s)][layer]
            Kc.append(k[r])
            Vc.append(v[r])
            o[r] = attention_decode(q[r], Kc.arr, Vc.arr, weight_round=self.wrnd)   # over L_i + 1 tokens
        attn = self.rnd(o.reshape(b, Hq * d)) @ W["wo"]
        x = x + attn
        xn2 = self.rnd(rmsnorm(x, W["g2"], self.eps))
        a = self.rnd(silu(xn2 @ W["wg"]) * (xn2 @ W["wu"]))
        ffn = a @ W["wd"]
        x = x + ffn
        return x, dict(attn=attn, ffn=ffn)

    def decode_step(self, mb, x: np.ndarray, seqs=None):
        """Run all layers on micro-batch mb.  x [b, h] (row r belongs to seqs[r]).

        seqs defaults to 0..b-1.  Rows are independent, so evaluating a subset
        of a micro-batch's sequences gives those rows of the full result.
        Returns (out [b, h], per_layer [n_layers, b, h]).
        """
        x = np.ascontiguousarray(x, dtype=self.dt)
        if seqs is None:
            seqs = list(range(x.shape[0]))
        assert len(seqs) == x.shape[0]
        per_layer = np.empty((self.nl,) + x.shape, dtype=self.dt)
        for l in range(self.nl):
            x, _ = self.layer_decode(l, mb, seqs, x)
            per_layer[l] = x
        return x, per_layer
