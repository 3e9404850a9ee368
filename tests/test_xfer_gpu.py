"""Transfer orchestrator on the GPU: data integrity in both directions, stream ordering through
pipemax_xfer_stream_wait, and an urgent copy overtaking queued KV-sized traffic."""
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_bulk_and_urgent_copies_arrive_intact_and_in_stream_order():
    import torch
    assert torch.cuda.is_available()
    from paper_2605_02189_amd import binding as pm
    x = pm.Xfer(device=0, max_inflight_bulk=2, chunk_bytes=1 << 20, log_capacity=1024)
    g = torch.Generator().manual_seed(0)
    n = (9 << 20) + 12345                                        # ragged tail: 9 whole chunks + a short one
    h_src = torch.randint(0, 256, (n,), dtype=torch.uint8, generator=g).pin_memory()
    d_buf = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    h_back = torch.zeros(n, dtype=torch.uint8).pin_memory()
    u_src = torch.randint(0, 256, (4096,), dtype=torch.uint8, generator=g).pin_memory()
    u_dev = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    t1 = x.submit(pm.XFER_BULK, pm.XFER_H2D, d_buf.data_ptr(), h_src.data_ptr(), n)
    t2 = x.submit(pm.XFER_URGENT, pm.XFER_H2D, u_dev.data_ptr(), u_src.data_ptr(), 4096)
    # a consumer stream waits for the bulk request, then reads the buffer
    s = torch.cuda.Stream()
    x.stream_wait(t1, s.cuda_stream)
    with torch.cuda.stream(s):
        total = d_buf.to(torch.int64).sum()
    x.wait(t2)
    assert torch.equal(u_dev.cpu(), u_src)
    s.synchronize()
    assert int(total) == int(h_src.to(torch.int64).sum())
    # and back: device -> host, cut into chunks, after the upload has completed
    x.wait(t1)
    t3 = x.submit(pm.XFER_BULK, pm.XFER_D2H, h_back.data_ptr(), d_buf.data_ptr(), n)
    x.wait(t3)
    assert torch.equal(h_back, h_src)
    log = x.log()
    up = [(o, b) for t, o, b, k, d in log if t == t1]
    assert up == [(i << 20, min(1 << 20, n - (i << 20))) for i in range(10)]
    st = x.stats()
    assert st["requests"] == {"urgent": 1, "bulk": 2} and st["chunks"]["bulk"] == 20
    x.drain()
    x.destroy()


def test_urgent_copy_does_not_wait_for_queued_kv_traffic():
    """2 GiB of bulk host-to-device traffic is queued (about 38 ms on this link); urgent 512 KiB copies in each
    direction submitted meanwhile complete in well under a millisecond each (median), long before the bulk."""
    import torch
    from paper_2605_02189_amd import binding as pm
    x = pm.Xfer(device=0, max_inflight_bulk=2, chunk_bytes=16 << 20)
    nb = 1 << 30
    h = torch.empty(nb, dtype=torch.uint8).pin_memory()
    h.fill_(3)
    d = torch.empty(nb, dtype=torch.uint8, device="cuda:0")
    a_h = torch.full((512 << 10,), 9, dtype=torch.uint8).pin_memory()
    a_d = torch.zeros(512 << 10, dtype=torch.uint8, device="cuda:0")
    b_h = torch.zeros(512 << 10, dtype=torch.uint8).pin_memory()
    b_d = torch.full((512 << 10,), 5, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    for _ in range(3):                                            # first use of the urgent streams: set-up cost
        x.wait(x.submit(pm.XFER_URGENT, pm.XFER_H2D, a_d.data_ptr(), a_h.data_ptr(), a_h.numel()))
        x.wait(x.submit(pm.XFER_URGENT, pm.XFER_D2H, b_h.data_ptr(), b_d.data_ptr(), b_h.numel()))
    a_d.zero_()
    b_h.zero_()
    torch.cuda.synchronize()
    x.submit(pm.XFER_BULK, pm.XFER_H2D, d.data_ptr(), h.data_ptr(), nb)
    tb = x.submit(pm.XFER_BULK, pm.XFER_H2D, d.data_ptr(), h.data_ptr(), nb)
    lats = []
    for _ in range(12):
        time.sleep(0.001)
        t0 = time.perf_counter()
        tu1 = x.submit(pm.XFER_URGENT, pm.XFER_H2D, a_d.data_ptr(), a_h.data_ptr(), a_h.numel())
        tu2 = x.submit(pm.XFER_URGENT, pm.XFER_D2H, b_h.data_ptr(), b_d.data_ptr(), b_h.numel())
        x.wait(tu1)
        x.wait(tu2)
        lats.append(time.perf_counter() - t0)
    still_running = not x.poll(tb)
    x.wait(tb)
    print("urgent pairs (ms):", [round(v * 1e3, 3) for v in lats], "bulk still running:", still_running, flush=True)
    assert bool((a_d == 9).all()) and bool((b_h == 5).all())
    assert bool((d[:: 1 << 16] == 3).all())
    assert still_running
    assert float(np.median(lats)) < 0.003                         # one or two 16 MiB chunks ahead, not 2 GiB
    x.destroy()


@pytest.mark.parametrize("config", ["C1_fp32", "mid_bf16"])
def test_stage_prefetch_through_the_orchestrator_keeps_parity(config):
    """The cyclic schedule with every prefetch copy cut into small chunks and issued by the orchestrator:
    same bars as the direct path (stage oracle on every step, bit-exact replica)."""
    import torch
    from test_parity_gpu import _check_replica, _mid_shape, _ragged_ctx, _run_cyclic_and_compare
    from helpers import check_tables
    from paper_2605_02189_amd import binding as pm
    from paper_2605_02189_amd.harness import StageRunner
    from paper_2605_02189_amd.synth_inputs import CONFIGS, SynthInputs
    if config == "C1_fp32":
        shape, tol, told, ctx = CONFIGS["C1"], 1e-5, 2e-4, None
    else:
        shape, tol, told = _mid_shape(), 1e-2, 3e-2
    syn = SynthInputs(shape, seed=41, pool_elems=1 << 23, gain_jitter=0.1)
    if config != "C1_fp32":
        ctx = _ragged_ctx(shape, syn)
    runner = StageRunner(shape, syn, flags=pm.FLAG_CAPTURE_LAYERS, ctx_lens=ctx).load()
    x = pm.Xfer(device=0, max_inflight_bulk=2, chunk_bytes=64 << 10, log_capacity=16)
    runner.stage.attach_xfer(x)
    orc = _run_cyclic_and_compare(runner, syn, shape, shape.decode_steps, tol_layer=tol, tol_delta=told)
    check_tables(runner)
    _check_replica(runner, syn, shape, orc, tol_new=tol)
    st = x.stats()
    assert st["bytes"]["bulk"] == runner.stage.get_stats()["h2d_bytes"] > 0
    assert st["chunks"]["bulk"] > st["requests"]["bulk"]          # the runs were cut
    runner.stage.attach_xfer(None)
    runner.stage.destroy()
    x.destroy()
