"""GPU test of the engine-driven training loop (the paper's Dependency Chaining
listing): producers on a second stream, pushes chained on the store's variable.
Values must match the oracle bit for bit, whatever the worker threads do."""
from __future__ import annotations

import numpy as np
import pytest

import workloads as wl
from tests.gpu_harness import Pair

pytestmark = pytest.mark.gpu
F = np.float32


@pytest.mark.parametrize("threads", [1, 4])
@pytest.mark.parametrize("cfg_id,descending", [(2, True), (2, False), (1, True)])
def test_engine_driven_steps_match_the_oracle(threads, cfg_id, descending):
    import torch
    from paper_1802_06949_amd.engine import Engine
    from paper_1802_06949_amd.training_loop import EngineLoop
    cfg = wl.get_config(cfg_id)
    K, W = len(cfg.keys), cfg.W
    pair = Pair(cfg.numel, W, "f32", cfg.bucket_bytes, lr=cfg.lr, momentum=cfg.momentum, wd=cfg.wd, descending=descending)
    eng = Engine(threads)
    side = torch.cuda.Stream()                                   # default priority
    loop = None
    try:
        pair.set_weights(wl.make_weights(cfg))
        live = [torch.zeros((W, n), dtype=torch.float32, device="cuda") for n in cfg.numel]
        staged = [torch.empty((W, n), dtype=torch.float32, device="cuda") for n in cfg.numel]
        loop = EngineLoop(pair.gpu, eng, staged, live, side.cuda_stream, [50] * K)
        for t in range(3):
            grads = wl.make_step_gradients(cfg, t)
            for k in range(K):
                staged[k].copy_(torch.from_numpy(np.stack(grads[k])))
            torch.cuda.synchronize()
            loop.step()
            pair.gpu.wait()
            pair.cpu.step(grads)
            pair.compare(f"engine step {t}")
        total, log = pair.gpu.launch_log()
        U = pair.gpu.plan.num_units
        if descending:
            # gradients arrive last layer first and the chain runs the same way: one launch per unit
            assert log == [(u, 1) for u in range(U - 1, -1, -1)] * 3
        else:
            # ascending chain: nothing can launch before key 0 is in, then everything goes at once
            assert log == [(0, U)] * 3
        assert eng.stats()[0] == 3 * 2 * K
    finally:
        if loop is not None:
            loop.close()
        eng.close()
        pair.close()


def test_stream_mix_diagnostic_sums_its_read_buffers():
    """kv_stream_mix (the measured ceiling for mixes of streams): every written buffer receives the sum, in buffer
    order, of the read buffers; bad shapes are refused."""
    import torch
    import paper_1802_06949_amd as kv
    n = 3 * 1024 + 8                                     # floats: several 4 KB tiles and a ragged one
    rng = np.random.Generator(np.random.SFC64([77, 1]))
    for n_read, n_write in ((1, 1), (2, 3), (4, 0), (8, 2), (16, 1), (32, 8)):
        host = [rng.standard_normal(n).astype(np.float32) for _ in range(n_read)]
        rd = [torch.from_numpy(h).cuda() for h in host]
        wr = [torch.full((n,), 7.0, device="cuda") for _ in range(n_write)]
        kv.stream_mix(rd, wr, n * 4)
        torch.cuda.synchronize()
        want = host[0].copy()
        for h in host[1:]:
            want = want + h                              # float32, left to right, as the kernel adds
        for w in wr:
            assert np.array_equal(w.cpu().numpy().view(np.uint32), want.view(np.uint32))
        for h, d in zip(host, rd):
            assert np.array_equal(d.cpu().numpy(), h)    # read buffers untouched
    a = torch.zeros(64, device="cuda")
    for bad in (([a] * 3, [a]), ([a], [a] * 9), ([], [a])):
        with pytest.raises(kv.KVError):
            kv.stream_mix(bad[0], bad[1], 256)
    with pytest.raises(kv.KVError):
        kv.stream_mix([a], [a], 250)                     # not a multiple of 16
