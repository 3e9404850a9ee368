"""Where the bf16 parity bar sits relative to what bf16 matrix-core operands can deliver at all.

The GPU path keeps the residual stream, all accumulators and the softmax statistics in fp32; what it cannot avoid
is rounding the two A operands of the FFN GEMMs to bf16 (the normalised activations and the SwiGLU output).  This
CPU test emulates exactly those two roundings on the oracle's own FFN arithmetic (attention left out: with
1024-token random prompts its update is a few per cent of the FFN's) for the ten first layers' worth of the 8B-shaped
benchmark stage's synthetic FFN weights (N(0, 0.02), the seeded generator the GPU tests use), and records how the relative L2 distance to the
fp32 result grows with depth.  It is the reason the accumulated-stream bar of the GPU parity tests is the larger of 1e-2 and
1.5 times the floor the oracle's operand-rounding mode finds on the same rows, while each layer on its own is held to
1e-2 at any depth."""
import numpy as np

from oracle.stage_oracle import rmsnorm, silu
from paper_2605_02189_amd.synth_inputs import CONFIGS, SynthInputs, bf16_bits_to_f32, to_bf16_bits


def _bf16(x):
    return bf16_bits_to_f32(to_bf16_bits(x))


def test_operand_rounding_alone_approaches_the_bar_with_depth():
    shape = CONFIGS["C2"].with_(n_layers=10)
    h, F, n_layers, rows = shape.hidden, shape.ffn, shape.n_layers, 2
    syn = SynthInputs(shape, seed=0)
    g = np.ones(h, dtype=np.float32)
    x_ref = syn.as_f32(syn.hidden(0, rows)).copy()
    x_emu = x_ref.copy()
    err, ratio = [], []
    for l in range(n_layers):
        wgu = syn.as_f32(syn._matrix("wgu", l, h, 2 * F))
        wd = syn.as_f32(syn._matrix("wd", l, F, h))
        outs = []
        for x, rnd in ((x_ref, lambda a: a), (x_emu, _bf16)):
            xn = rnd(rmsnorm(x, g, 1e-5))
            gu = xn @ wgu
            upd = rnd(silu(gu[:, :F]) * gu[:, F:]) @ wd
            outs.append((x + upd, float(np.linalg.norm(upd) / np.linalg.norm(x))))
        (x_ref, r), (x_emu, _) = outs
        ratio.append(r)
        err.append(float(np.linalg.norm(x_emu - x_ref) / np.linalg.norm(x_ref)))
    print("update / stream:", [round(r, 2) for r in ratio])
    print("rel L2 after each layer:", [f"{e:.2e}" for e in err])
    assert ratio[0] > 1.5 and min(ratio) > 0.25       # updates as large as the stream they join: nothing is diluted
    assert all(b > a for a, b in zip(err, err[1:]))   # so the error is handed on undiluted and grows monotonically
    assert 1.5e-3 < err[0] < 5e-3                     # one layer: a few 1e-3
    assert 5e-3 < err[7] < 1e-2                       # 8 layers: inside the bar, most of it used up
    assert err[9] > 0.7e-2                            # 10 layers: at the bar's doorstep before any other rounding
