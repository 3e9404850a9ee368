"""Seeded synthetic inputs and the workload shapes.

This module serves both the HIP path (through tests and bench.py) and the CPU
oracle.  It holds none of the method's arithmetic: only shapes, random number
draws and the float32 -> bfloat16 storage rounding of the generated values.

Recipe.  Two master pools of normal deviates are drawn once per seed: N(0, 1)
for cached K, V and hidden states, N(0, 0.02) for weight matrices.  Every tensor
is cut from its pool at offsets drawn from a generator seeded by
(seed, tensor kind, indices), one offset per tensor (K, V, hidden) or per row
(weight matrices, which can be larger than the pool).  This keeps the value
distribution of the workload while making the 10-GB to 100-GB pools of the
larger configurations a matter of memory copies.  RMSNorm gains are 1.

The shapes are those of the benchmark configurations; they stand in for the
request-length mixes of the ShareGPT and LongBench workloads the paper measures
on (Table 2), whose items are not used.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class StageShape:
    name: str
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    dtype: str              # "fp32" | "bf16"
    rope_base: float
    n_microbatches: int
    seqs_per_mb: int
    ctx_lo: int             # prompt length, uniform on [ctx_lo, ctx_hi]
    ctx_hi: int
    decode_steps: int
    rms_eps: float = 1e-5
    page_tokens: int = 16

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "fp32" else 2

    @property
    def n_qkv(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_layers * self.n_kv_heads * self.head_dim * self.elem_bytes

    @property
    def page_bytes(self) -> int:
        return self.page_tokens * self.kv_bytes_per_token

    @property
    def weight_bytes(self) -> int:
        per_layer = (self.hidden * self.n_qkv + self.n_q_heads * self.head_dim * self.hidden
                     + 3 * self.hidden * self.ffn)
        return self.n_layers * per_layer * self.elem_bytes

    def with_(self, **kw) -> "StageShape":
        return replace(self, **kw)


CONFIGS = {
    # configs[0]: tiny fp32 stage the oracle runs in full
    "C1": StageShape("C1", 2, 256, 4, 2, 64, 688, "fp32", 10000.0, 4, 8, 128, 128, 16),
    # configs[1]: 8 of 32 layers of an 8B-shaped model, uniform 1024-token prompts
    "C2": StageShape("C2", 8, 4096, 32, 8, 128, 14336, "bf16", 500000.0, 4, 64, 1024, 1024, 256),
    # configs[2]: same stage, ragged prompts
    "C3": StageShape("C3", 8, 4096, 32, 8, 128, 14336, "bf16", 500000.0, 6, 128, 512, 4096, 128),
    # configs[3]: 10 of 80 layers of a 70B-shaped model
    "C4": StageShape("C4", 10, 8192, 64, 8, 128, 28672, "bf16", 500000.0, 8, 256, 2048, 2048, 64),
    # configs[4]: memory-pressure stress on the same stage
    "C5": StageShape("C5", 10, 8192, 64, 8, 128, 28672, "bf16", 500000.0, 8, 256, 4096, 4096, 32),
}


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


_KIND = {"kv": 1, "hidden": 2, "wqkv": 3, "wo": 4, "wgu": 5, "wd": 6, "ctx": 7, "gain": 8}


class SynthInputs:
    """All inputs of one workload, reproducible from (shape, seed)."""

    def __init__(self, shape: StageShape, seed: int = 0, pool_elems: int = 1 << 25,
                 gain_jitter: float = 0.0):
        self.shape = shape
        self.seed = int(seed)
        self.gain_jitter = float(gain_jitter)   # parity tests use gains 1 + jitter*N(0,1)
        rng = np.random.default_rng([self.seed, 0])
        unit = rng.standard_normal(pool_elems, dtype=np.float32)
        wts = unit[::-1] * np.float32(0.02)          # reversed copy: a different sequence
        if shape.dtype == "bf16":
            self._unit = to_bf16_bits(unit)
            self._wts = to_bf16_bits(wts)
        else:
            self._unit = unit
            self._wts = np.ascontiguousarray(wts)
        self._n = pool_elems

    # storage dtype of every array handed out
    @property
    def np_dtype(self):
        return np.uint16 if self.shape.dtype == "bf16" else np.float32

    def as_f32(self, a: np.ndarray) -> np.ndarray:
        """Exact float32 view of the stored values (what both sides compute from)."""
        return bf16_bits_to_f32(a) if self.shape.dtype == "bf16" else np.asarray(a, dtype=np.float32)

    def _rng(self, kind: str, *idx):
        return np.random.default_rng([self.seed, _KIND[kind], *[int(i) for i in idx]])

    # -- lengths ------------------------------------------------------------
    def ctx_lens(self, mb: int) -> np.ndarray:
        s = self.shape
        if s.ctx_lo == s.ctx_hi:
            return np.full(s.seqs_per_mb, s.ctx_lo, dtype=np.int32)
        return self._rng("ctx", mb).integers(s.ctx_lo, s.ctx_hi + 1, size=s.seqs_per_mb).astype(np.int32)

    # -- cached K, V of a prompt -------------------------------------------
    def kv_prefix(self, mb: int, seq: int, layer: int, L: int):
        """(K, V), each [L, Hkv, d] in the stage's storage dtype; views of the pool."""
        s = self.shape
        n = L * s.n_kv_heads * s.head_dim
        assert n <= self._n
        off = self._rng("kv", mb, seq, layer).integers(0, self._n - n + 1, size=2)
        shp = (L, s.n_kv_heads, s.head_dim)
        return (self._unit[off[0]: off[0] + n].reshape(shp),
                self._unit[off[1]: off[1] + n].reshape(shp))

    # -- hidden states entering the stage ------------------------------------
    def hidden(self, step: int, b: int) -> np.ndarray:
        n = b * self.shape.hidden
        off = int(self._rng("hidden", step).integers(0, self._n - n + 1))
        return self._unit[off: off + n].reshape(b, self.shape.hidden)

    # -- weights ------------------------------------------------------------
    def _matrix(self, kind: str, layer: int, rows: int, cols: int) -> np.ndarray:
        offs = self._rng(kind, layer).integers(0, self._n - cols + 1, size=rows)
        out = np.empty((rows, cols), dtype=self.np_dtype)
        for r in range(rows):
            out[r] = self._wts[offs[r]: offs[r] + cols]
        return out

    def weights(self, layer: int) -> dict:
        s = self.shape
        def gain(which):
            g = np.ones(s.hidden, dtype=np.float32)
            if self.gain_jitter:
                g += np.float32(self.gain_jitter) * self._rng("gain", layer, which).standard_normal(
                    s.hidden, dtype=np.float32)
            return to_bf16_bits(g) if s.dtype == "bf16" else g
        return dict(
            wqkv=self._matrix("wqkv", layer, s.hidden, s.n_qkv),
            wo=self._matrix("wo", layer, s.n_q_heads * s.head_dim, s.hidden),
            wgu=self._matrix("wgu", layer, s.hidden, 2 * s.ffn),
            wd=self._matrix("wd", layer, s.ffn, s.hidden),
            g1=gain(1), g2=gain(2))
