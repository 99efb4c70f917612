"""GPU parity of the funneled and concurrent schedules (the paper's "MPI Funneled"
and "MPI Concurrent Communications" designs) against the same oracle: the three
schedules differ in when and where a key's aggregation runs, never in its value."""
from __future__ import annotations

import numpy as np
import pytest

import workloads as wl
from oracle import kv_oracle as orc
from tests.gpu_harness import Pair, run_config

pytestmark = pytest.mark.gpu
F = np.float32
CHAINED, FUNNEL, CONCURRENT = 0, 1, 2


def _rng(*seed):
    return np.random.Generator(np.random.SFC64(list(seed)))


def _grads(numel, W, dtype, seed):
    out = []
    for k, n in enumerate(numel):
        gk = [(_rng(seed, k, r).standard_normal(n, dtype=F) * F(0.01)).astype(F) for r in range(W)]
        out.append([g.astype(np.float16) for g in gk] if dtype == "f16" else gk)
    return out


SCHEDULES = [(FUNNEL, 1, 0), (CONCURRENT, 1, 0), (CONCURRENT, 3, 0), (CONCURRENT, 8, 2), (CONCURRENT, 4, 5)]


@pytest.mark.parametrize("schedule", SCHEDULES, ids=lambda s: f"sched{s[0]}-n{s[1]}-o{s[2]}")
@pytest.mark.parametrize("mode", ["list", "each"])
def test_resnet20_under_every_schedule(schedule, mode):
    run_config(wl.get_config(2), 3, mode=mode, schedule=schedule, label=f"schedule {schedule}")


@pytest.mark.parametrize("schedule", SCHEDULES, ids=lambda s: f"sched{s[0]}-n{s[1]}-o{s[2]}")
@pytest.mark.parametrize("dtype,order", [("f32", orc.PAIRWISE), ("f16", orc.SEQUENTIAL)])
def test_ragged_keys_under_every_schedule(schedule, dtype, order):
    numel = [0, 1, 5, 64, 1023, 1025, 4096, 4099, 0, 20000, 7]
    pair = Pair(numel, 5, dtype, 8192, lr=0.1, momentum=0.9, wd=1e-4, order=order, schedule=schedule)
    try:
        pair.set_weights([_rng(1, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        for t in range(3):
            pair.step(_grads(numel, 5, dtype, 10 + t), mode="each", order=[int(x) for x in _rng(2, t).permutation(len(numel))])
            pair.compare(f"{schedule} step {t}")
    finally:
        pair.close()


@pytest.mark.timeout(300)
@pytest.mark.parametrize("schedule", [(FUNNEL, 1, 0), (CONCURRENT, 4, 8)], ids=["funnel", "concurrent"])
def test_resnet50_full_size_per_key_schedules(schedule):
    run_config(wl.get_config(3), 2, keep_sum=False, gen_threads=16, oracle_threads=8, schedule=schedule)


def test_per_key_launches_follow_the_push_order():
    numel = [100, 0, 5000, 64, 3000]
    pair = Pair(numel, 2, "f32", 1 << 20, lr=0.1, momentum=0.0, wd=0.0, schedule=(FUNNEL, 1, 0))
    try:
        g = _grads(numel, 2, "f32", 20)
        order = [4, 1, 0, 3, 2]
        pair.step(g, mode="each", order=order)
        total, log = pair.gpu.launch_log()
        assert log == [(k, 0) for k in order if numel[k] > 0] and total == 4    # the empty key launches nothing
        pair.compare("funnel order")
    finally:
        pair.close()


def test_switching_schedules_between_iterations():
    numel = [100, 5000, 64, 3000, 9]
    W = 4
    pair = Pair(numel, W, "f32", 4096, lr=0.1, momentum=0.9, wd=1e-4)
    try:
        pair.set_weights([_rng(3, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        seq = [(CHAINED, 1, 0), (FUNNEL, 1, 0), (CONCURRENT, 3, 2), (CHAINED, 1, 0), (CONCURRENT, 2, 0), (FUNNEL, 1, 0)]
        for t, sched in enumerate(seq):
            pair.gpu.set_schedule(*sched)
            pair.step(_grads(numel, W, "f32", 30 + t), mode="each" if t % 2 else "list")
            pair.compare(f"after switching to {sched}")
        # a switch in the middle of a chained iteration is refused
        pair.gpu.set_schedule(CHAINED)
        dev = pair.upload(_grads(numel, W, "f32", 40))
        pair.gpu.push(0, dev[0])
        with pytest.raises(pair.kv.KVError) as e:
            pair.gpu.set_schedule(FUNNEL)
        assert e.value.status == -3
        with pytest.raises(pair.kv.KVError):
            pair.gpu.set_schedule(CONCURRENT, 0, 0)
        with pytest.raises(pair.kv.KVError):
            pair.gpu.set_schedule(7)
    finally:
        pair.close()


def test_concurrent_pull_then_barrier_sees_the_update():
    import torch
    numel = [4096, 4096, 4096]
    pair = Pair(numel, 2, "f32", 1 << 20, lr=0.5, momentum=0.0, wd=0.0, schedule=(CONCURRENT, 3, 0))
    try:
        g = _grads(numel, 2, "f32", 50)
        dev = pair.upload(g)
        outs = [torch.zeros(n, device="cuda") for n in numel]
        for k in range(3):
            pair.gpu.push(k, dev[k])
            pair.gpu.pull(k, outs[k])               # on the key's stream, after its update
        pair.gpu.barrier()
        pair.cpu.step(g)
        for k in range(3):
            assert np.array_equal(outs[k].cpu().numpy(), pair.cpu.w[k])
    finally:
        pair.close()


@pytest.mark.parametrize("schedule", [(CONCURRENT, 4, 0), (CHAINED, 1, 0)], ids=["concurrent", "chained"])
def test_wait_for_one_key_covers_its_launch_and_its_pulls(schedule):
    """kv_wait(key) waits for the event of that key's last launch (or of a pull issued after it), not for the
    stream: what the key's pull wrote must be complete when it returns, under per-key launches on several
    streams and under per-unit launches on one stream."""
    import torch
    numel = [1 << 20, 300, 1 << 19, 70000, 5, 1 << 20]
    pair = Pair(numel, 4, "f32", 64 << 10, lr=0.5, momentum=0.9, wd=0.0, schedule=schedule)
    try:
        pair.set_weights([_rng(60, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        host = [torch.empty(n, dtype=torch.float32).pin_memory() for n in numel]
        for t in range(3):
            g = _grads(numel, 4, "f32", 61 + t)
            dev = pair.upload(g)
            outs = [torch.zeros(n, device="cuda") for n in numel]
            torch.cuda.synchronize()
            for k in range(len(numel)):
                pair.gpu.push(k, dev[k])
                pair.gpu.pull(k, outs[k])
            pair.cpu.step(g)
            side = torch.cuda.Stream()
            for k in reversed(range(len(numel))):
                pair.gpu.wait(k)
                with torch.cuda.stream(side):          # a stream that is ordered after nothing of the store's
                    host[k].copy_(outs[k], non_blocking=True)
                side.synchronize()
                assert np.array_equal(host[k].numpy().view(np.uint32), pair.cpu.w[k].view(np.uint32)), f"step {t} key {k}"
            pair.gpu.wait()
    finally:
        pair.close()


def test_small_launches_share_completion_events_and_a_large_one_gets_its_own():
    """A stream records a completion event after every 8th launch that may be waited for, or once 64 MB of launch
    traffic have gone out since its last one; kv_wait(key) waits for the first event of the key's stream at or after
    the key's launch, else for the stream.  Two streams: key 0 (4 ranks of 3M floats and the state: 96 MB) and twenty
    small keys on the first, twenty small keys on the second."""
    import torch
    numel = [3 << 20] + [776 + 12 * k for k in range(40)]
    W = 4
    pair = Pair(numel, W, "f32", 64 << 10, lr=0.5, momentum=0.9, wd=0.0, schedule=(CONCURRENT, 2, 0))
    try:
        pair.set_weights([_rng(70, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        arena = [type("P", (), {"data_ptr": lambda self, p=pair.gpu.weights_ptr(k): p})() for k in range(len(numel))]
        outs = [torch.zeros(n, device="cuda") for n in numel]
        side = torch.cuda.Stream()                     # a stream that is ordered after nothing of the store's
        recorded = pair.gpu.completion_events()
        for t in range(2):
            g = _grads(numel, W, "f32", 71 + t)
            dev = pair.upload(g)
            torch.cuda.synchronize()
            for k in range(len(numel)):
                pair.gpu.push(k, dev[k])
            # first stream: key 0 by its bytes, then the 8th and 16th of the twenty after it; second stream: its
            # 8th and 16th (the counts carry over from one step to the next: 20 more marks, 2 or 3 more events)
            now = pair.gpu.completion_events()
            assert 5 <= now - recorded <= 6, (t, now - recorded)
            recorded = now
            pair.cpu.step(g)
            for k in reversed(range(len(numel))):
                pair.gpu.wait(k)
                pair.kv.copy_bytes(outs[k], arena[k], numel[k] * 4, stream=side.cuda_stream)
                side.synchronize()
                assert np.array_equal(outs[k].cpu().numpy().view(np.uint32), pair.cpu.w[k].view(np.uint32)), f"step {t} key {k}"
            assert pair.gpu.completion_events() == recorded     # waiting records nothing
            pair.gpu.wait()
    finally:
        pair.close()


def test_lazy_store_merges_single_pushes_into_one_launch():
    """The paper's Dependency Chaining loop: all pushes first, then the pulls.  With
    KV_FLAG_LAZY_LAUNCH the single pushes pile up and the whole iteration is one launch."""
    import torch
    cfg = wl.get_config(2)
    K = len(cfg.keys)
    pair = Pair(cfg.numel, cfg.W, "f32", cfg.bucket_bytes, lr=cfg.lr, momentum=cfg.momentum, wd=cfg.wd, lazy=True)
    try:
        U = pair.gpu.plan.num_units
        pair.set_weights(wl.make_weights(cfg))
        for t in range(2):
            pair.step(wl.make_step_gradients(cfg, t), mode="each", order=[int(x) for x in _rng(60 + t).permutation(K)])
            pair.compare(f"lazy step {t}")
        assert pair.gpu.launch_log()[1] == [(0, U)] * 2
        # a pull in the middle of the pushes launches what is ready and is served after its key's update
        g = wl.make_step_gradients(cfg, 2)
        dev = pair.upload(g)
        first_unit_keys = pair.gpu.plan.unit(0)[0]
        for k in first_unit_keys:
            pair.gpu.push(k, dev[k])
        assert pair.gpu.launch_log()[0] == 2                   # nothing launched yet
        out = torch.zeros(cfg.numel[first_unit_keys[0]], device="cuda")
        pair.gpu.pull(first_unit_keys[0], out)
        assert pair.gpu.launch_log()[1][-1] == (0, 1)          # unit 0 went out for the pull
        for k in range(K):
            if k not in first_unit_keys:
                pair.gpu.push(k, dev[k])
        # the last push of the iteration launches the rest itself: it does not wait for a pull or a wait
        assert pair.gpu.launch_log()[0] == 4 and pair.gpu.launch_log()[1][-1] == (1, U - 1)
        pair.gpu.wait()
        pair.cpu.step(g)
        assert np.array_equal(out.cpu().numpy(), pair.cpu.w[first_unit_keys[0]])
        pair.compare("lazy with a pull in the middle")
        assert pair.gpu.launch_log()[1][-1] == (1, U - 1)
    finally:
        pair.close()
