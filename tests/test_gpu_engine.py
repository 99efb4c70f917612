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
