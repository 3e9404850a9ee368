"""Driver of the stage library for tests, smoke() and bench.py: builds a stage from a workload
shape and its synthetic inputs and runs the cyclic schedule of Eq. 3 (execute D_i, prefetch D_j,
overwrite D_k).  PyTorch is used for the hidden-state device buffers and the compute stream only.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as pm
from .synth_inputs import StageShape, SynthInputs


def pages_for(tokens: int, page_tokens: int = 16) -> int:
    return -(-int(tokens) // page_tokens)


class StageRunner:
    """One stage + its micro-batches.

    sigma = streamed fraction of every micro-batch: the last round(sigma*b) sequences of each
    micro-batch are evicted after their step and prefetched before their next one; the others stay
    GPU-resident (the hybrid resident + prefetched composition of Sec. 3.1.2).
    """

    def __init__(self, shape: StageShape, syn: SynthInputs, *, sigma: float = 1.0, steps: int | None = None,
                 flags: int = 0, device: int = 0, n_microbatches: int | None = None,
                 ctx_lens: dict | None = None, gpu_pool_all_resident: bool = False,
                 wb_layers_per_copy: int = 0, reserve: bool = True, gpu_pages: int | None = None,
                 max_rows: int | None = None, real_microbatches: int | None = None,
                 gpu_resident_microbatches: int | None = None, arenas: int = 2):
        """real_microbatches = r < n: only micro-batches 0..r-1 get host pages and KV of their own; micro-batch
        m >= r is an alias of m mod r (same lengths, same host pages; hosts that cannot pin the whole
        configuration; timing only).  gpu_resident_microbatches: size the GPU pool for that many whole
        micro-batches (compute-only legs of configurations whose KV exceeds the HBM).
        arenas: GPU room for that many streamed parts.  2 = the schedule of Eq. 3: the prefetch of D_{i+1} overwrites
        D_{i-1}, so it can start only when step t-1 has ended and has exactly the length of step t to finish.
        3 = D_{i-1} stays one iteration longer and the prefetch overwrites D_{i-2}, whose last step ended long ago:
        the copy no longer waits for the compute stream at all (needs n >= 4 micro-batches)."""
        self.shape, self.syn = shape, syn
        pool_override = gpu_pages
        self.n = n_microbatches or shape.n_microbatches
        self.arenas = 3 if (arenas >= 3 and self.n >= 4) else 2
        self.n_real = min(self.n, real_microbatches or self.n)
        self.b = shape.seqs_per_mb
        self.steps = steps if steps is not None else shape.decode_steps
        self.device = device
        self.ctx0 = {mb: np.asarray(ctx_lens[mb] if ctx_lens else syn.ctx_lens(mb), dtype=np.int32)
                     for mb in range(self.n_real)}
        for mb in range(self.n_real, self.n):
            self.ctx0[mb] = self.ctx0[mb % self.n_real]
        self.b_of = {mb: len(self.ctx0[mb]) for mb in range(self.n)}
        steps_per_mb = -(-self.steps // self.n)
        grow = pages_for(steps_per_mb) + 1
        self._set_sigma(sigma)
        full = {mb: [pages_for(l) + grow for l in self.ctx0[mb]] for mb in range(self.n)}
        host_pages = sum(sum(full[mb]) for mb in range(self.n_real))
        all_pages = sum(sum(v) for v in full.values())
        resident_pages = sum(sum(full[mb][: self.b_of[mb] - self.n_stream[mb]]) for mb in range(self.n))
        stream_pages = sorted((sum(full[mb][self.b_of[mb] - self.n_stream[mb]:]) for mb in range(self.n)),
                              reverse=True)
        gpu_pages = resident_pages + sum(stream_pages[:self.arenas]) + 8     # arenas for the streamed part
        if gpu_pool_all_resident:                                       # room to keep everything on the GPU
            gpu_pages = all_pages + 8
        if gpu_resident_microbatches is not None:
            gpu_pages = max(gpu_pages, sum(sorted((sum(v) for v in full.values()), reverse=True)
                                           [:gpu_resident_microbatches]) + 8)
        if pool_override is not None:                                   # caller-chosen GPU pool (scheduler runs)
            gpu_pages = int(pool_override)
        max_ctx = int(max(int(c.max()) for c in self.ctx0.values())) + steps_per_mb + 1
        self.max_ctx = max_ctx
        self.reserve_tokens = (steps_per_mb + 1) if reserve else 0
        self.stage = pm.Stage(
            n_layers=shape.n_layers, hidden=shape.hidden, n_q_heads=shape.n_q_heads,
            n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, ffn=shape.ffn,
            rope_base=shape.rope_base, rms_eps=shape.rms_eps,
            dtype=pm.F32 if shape.dtype == "fp32" else pm.BF16, n_microbatches=self.n,
            max_seqs_per_mb=max(max(self.b_of.values()), max_rows or 0), max_ctx=max_ctx,
            gpu_kv_bytes=gpu_pages * shape.page_bytes, host_kv_bytes=(host_pages + 8) * shape.page_bytes,
            device=device, flags=flags, host_reserve_tokens=self.reserve_tokens,
            wb_layers_per_copy=wb_layers_per_copy)
        self.torch_dtype = torch.float32 if shape.dtype == "fp32" else torch.bfloat16
        self.t = 0

    def _set_sigma(self, sigma: float):
        self.sigma = float(sigma)
        self.n_stream = {mb: int(round(sigma * self.b_of[mb])) for mb in range(self.n)}
        self.stream_ids = {mb: np.arange(self.b_of[mb] - self.n_stream[mb], self.b_of[mb], dtype=np.int32)
                           for mb in range(self.n)}

    def restart(self, sigma: float):
        """Changes the streamed fraction and restarts the cycle at iteration 0: the sequences that are streamed from
        now on leave the GPU, the others come (or stay) resident.  Needs a GPU pool that can hold the resident
        parts plus two streamed parts."""
        self.stage.sync()
        self._set_sigma(sigma)
        for mb in range(self.n):
            if self.n_stream[mb]:
                self.stage.evict_kv(mb, self.stream_ids[mb])
        self.stage.sync()
        self.t = 0
        self.warm_start()
        self.stage.sync()

    # -- set-up ---------------------------------------------------------------------------------
    def load_weights(self):
        for l in range(self.shape.n_layers):
            w = self.syn.weights(l)
            self.stage.set_weight(l, pm.W_QKV, w["wqkv"])
            self.stage.set_weight(l, pm.W_O, w["wo"])
            self.stage.set_weight(l, pm.W_GU, w["wgu"])
            self.stage.set_weight(l, pm.W_D, w["wd"])
            self.stage.set_weight(l, pm.G_ATTN, w["g1"])
            self.stage.set_weight(l, pm.G_FFN, w["g2"])

    def load_kv(self):
        for mb in range(self.n_real):
            self.stage.mb_define(mb, self.ctx0[mb])
            for s, L in enumerate(self.ctx0[mb]):
                if L == 0:
                    continue
                for l in range(self.shape.n_layers):
                    K, V = self.syn.kv_prefix(mb, s, l, int(L))
                    self.stage.kv_host_write(mb, s, l, 0, K, V)
        for mb in range(self.n_real, self.n):
            self.stage.mb_define_alias(mb, mb % self.n_real)

    def load(self):
        self.load_weights()
        self.load_kv()
        return self

    # -- hidden states ----------------------------------------------------------------------------
    def hidden_tensor(self, step: int, mb: int) -> torch.Tensor:
        a = self.syn.hidden(step, self.b_of[mb])
        if self.shape.dtype == "bf16":
            t = torch.from_numpy(a.view(np.int16).copy()).view(torch.bfloat16)
        else:
            t = torch.from_numpy(np.array(a, dtype=np.float32))
        return t.to(f"cuda:{self.device}")

    def to_numpy_f32(self, t: torch.Tensor) -> np.ndarray:
        return t.float().cpu().numpy()

    # -- schedule ---------------------------------------------------------------------------------
    def warm_start(self):
        """Brings the resident parts of all micro-batches and all of D_0 onto the GPU."""
        for mb in range(self.n):
            nres = self.b_of[mb] - self.n_stream[mb]
            if nres:
                self.stage.prefetch_kv(mb, np.arange(nres, dtype=np.int32))
        self.stage.prefetch_kv(0)

    def step(self, hidden_in: torch.Tensor | None, hidden_out: torch.Tensor | None,
             stream: torch.cuda.Stream | None = None, transfers: bool = True, compute: bool = True):
        """Iteration t of the cyclic schedule: overwrite D_k, prefetch D_j, execute D_i (Eq. 3).  None of the
        three calls blocks on the GPU.  The transfers are arranged first: the prefetch worker then issues the
        copies the moment the last reader of the overwritten pages (step t-1) ends, while the host is still
        enqueuing step t; arranged after the step they start 0.2-0.3 ms later and, where a copy takes about as
        long as a step, no longer fit behind it.
        transfers=False keeps everything where it is (all micro-batches must be resident);
        compute=False issues only the evict / prefetch traffic of the iteration."""
        n, t = self.n, self.t
        lag = self.arenas - 1                      # the micro-batch that ran `lag` iterations ago is overwritten
        i, j, k = t % n, (t + 1) % n, (t - lag) % n
        if transfers:
            if t >= lag and self.n_stream[k] and k != i and k != j:
                self.stage.evict_kv(k, self.stream_ids[k])
            if j != i and self.n_stream[j]:
                self.stage.prefetch_kv(j, self.stream_ids[j])
        if compute:
            sp = stream.cuda_stream if stream is not None else torch.cuda.current_stream().cuda_stream
            self.stage.decode_step(i, hidden_in.data_ptr(), hidden_out.data_ptr(), sp)
        self.t += 1
        return i
