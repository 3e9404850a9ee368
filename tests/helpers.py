"""Shared pieces of the GPU parity tests: an oracle built from the same synthetic inputs."""
import numpy as np

from oracle.stage_oracle import StageOracle


def make_oracle(shape, syn, ctx0: dict, seqs: dict | None = None, dtype=np.float32,
                share_weights_of: StageOracle | None = None, operand_round=None) -> StageOracle:
    """ctx0[mb] = prompt lengths; seqs[mb] = which sequences to track (default all).  share_weights_of: another
    oracle of the same stage whose weight arrays this one reads too (the 70B-shaped stage is 34 GB in fp32)."""
    orc = StageOracle(shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                      shape.ffn, shape.rope_base, shape.rms_eps, dtype=dtype, operand_round=operand_round)
    for l in range(shape.n_layers):
        if share_weights_of is not None:
            orc.w[l] = share_weights_of.w[l]
            continue
        w = syn.weights(l)
        orc.set_layer_weights(l, **{k: syn.as_f32(v) for k, v in w.items()})
    for mb, lens in ctx0.items():
        for s in (seqs[mb] if seqs else range(len(lens))):
            kv = [syn.kv_prefix(mb, s, l, int(lens[s])) for l in range(shape.n_layers)]
            orc.define_sequence(mb, s, [syn.as_f32(k) for k, _ in kv], [syn.as_f32(v) for _, v in kv])
    return orc


def check_tables(runner, n_gpu_pages_total=None):
    """Block tables: right length, inside the pool, no page owned twice; both pools' free counts equal what the
    tables and the growth reservation account for.  (Micro-batches defined as aliases share their source's host
    pages by construction and are left out of the host-side checks.)"""
    st = runner.stage
    stats = st.get_stats()
    gpu_seen, host_seen = set(), set()
    host_held = 0
    n_real = getattr(runner, "n_real", runner.n)
    for mb in range(runner.n):
        lens = st.get_ctx_lens(mb)
        res = st.get_residency(mb)
        for s in range(runner.b_of[mb]):
            g, h = st.get_block_table(mb, s)
            assert len(h) == -(-int(lens[s]) // 16), (mb, s, len(h), lens[s])
            assert len(set(h.tolist())) == len(h)
            assert all(0 <= p < stats["host_pages_total"] for p in h)
            if mb < n_real:
                assert not (set(h.tolist()) & host_seen)
                host_seen |= set(h.tolist())
                # a sequence holds the pages reserved for it at definition (prompt + reserve, capped at max_ctx)
                # until it has outgrown them; from then on exactly the pages of its table
                reserved = -(-min(runner.max_ctx, int(runner.ctx0[mb][s]) + runner.reserve_tokens) // 16)
                host_held += max(reserved, len(h))
            if res[s] == 0:
                assert all(p == -1 for p in g)
            else:
                assert all(0 <= p < stats["gpu_pages_total"] for p in g)
                assert not (set(g.tolist()) & gpu_seen)
                gpu_seen |= set(g.tolist())
    assert stats["gpu_pages_free"] == stats["gpu_pages_total"] - len(gpu_seen)
    if n_real == runner.n:
        assert stats["host_pages_free"] == stats["host_pages_total"] - host_held
