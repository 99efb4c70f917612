"""GPU parity of the fused broadcast: the kernel that updates a key also writes the
new weights to every replica buffer (the third phase of the paper's collective).
fp32 replicas must equal the oracle's weights bit for bit, fp16 replicas the
oracle's round-to-nearest-even conversion of them."""
from __future__ import annotations

import numpy as np
import pytest

import workloads as wl
from oracle import kv_oracle as orc
from tests.gpu_harness import Pair, same_bits_or_both_nan

pytestmark = pytest.mark.gpu
F = np.float32


def _rng(*seed):
    return np.random.Generator(np.random.SFC64(list(seed)))


def _grads(numel, W, dtype, seed, scale=0.01):
    out = []
    for k, n in enumerate(numel):
        gk = [(_rng(seed, k, r).standard_normal(n, dtype=F) * F(scale)).astype(F) for r in range(W)]
        out.append([g.astype(np.float16) for g in gk] if dtype == "f16" else gk)
    return out


def _replicas(numel, R, dtype, misalign=0):
    import torch
    tdt = torch.float32 if dtype == "f32" else torch.float16
    reps = []
    for n in numel:
        row = []
        for _ in range(R):
            buf = torch.full((n + misalign + 8,), 7.0, dtype=tdt, device="cuda")
            row.append(buf[misalign:misalign + n])
        reps.append(row)
    return reps


def _check(pair, reps, dtype, label):
    for k, row in enumerate(reps):
        ref = pair.cpu.w[k] if dtype == "f32" else orc.round_to_half(pair.cpu.w[k])
        for r, t in enumerate(row):
            got = t.cpu().numpy()
            if dtype == "f32":
                assert same_bits_or_both_nan(got, ref), f"{label}: key {k} replica {r}"
            else:
                assert np.array_equal(got.view(np.uint16), ref.view(np.uint16)), f"{label}: key {k} replica {r}"


NUMEL = [0, 1, 5, 64, 1023, 1024, 1025, 4096, 4099, 0, 20000, 7]


@pytest.mark.parametrize("grad_dtype", ["f32", "f16"])
@pytest.mark.parametrize("rep_dtype", ["f32", "f16"])
@pytest.mark.parametrize("R", [1, 3, 8])
@pytest.mark.parametrize("schedule", [None, (1, 1, 0), (2, 3, 0)], ids=["chained", "funnel", "concurrent"])
def test_replicas_receive_the_updated_weights(grad_dtype, rep_dtype, R, schedule):
    W = 4
    pair = Pair(NUMEL, W, grad_dtype, 8192, lr=0.1, momentum=0.9, wd=1e-4, schedule=schedule)
    try:
        pair.set_weights([_rng(1, k).standard_normal(n, dtype=F) for k, n in enumerate(NUMEL)])
        reps = _replicas(NUMEL, R, rep_dtype)
        for k in range(len(NUMEL)):
            pair.gpu.set_broadcast(k, reps[k], rep_dtype)
        # the paper's KVStore.init: every worker receives the initial value
        pair.gpu.broadcast_weights()
        pair.gpu.wait()
        _check(pair, reps, rep_dtype, "initial value")
        for t in range(3):
            pair.step(_grads(NUMEL, W, grad_dtype, 10 + t), mode="list" if t != 1 else "each")
            pair.compare(f"step {t}")
            _check(pair, reps, rep_dtype, f"step {t}")
    finally:
        pair.close()


@pytest.mark.parametrize("rep_dtype,misalign", [("f32", 1), ("f32", 2), ("f16", 1), ("f16", 4)])
def test_replicas_that_are_not_16_byte_aligned(rep_dtype, misalign):
    numel = [5, 1000, 4096, 9001]
    pair = Pair(numel, 2, "f32", 1 << 20, lr=0.1, momentum=0.9, wd=1e-4)
    try:
        reps = _replicas(numel, 2, rep_dtype, misalign)
        pair.set_weights([_rng(2, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        for k in range(len(numel)):
            pair.gpu.set_broadcast(k, reps[k], rep_dtype)
        for k in (3, 1, 0, 2):                       # key by key
            pair.gpu.broadcast_weights(k)
        pair.gpu.wait()
        _check(pair, reps, rep_dtype, "misaligned initial value")
        for t in range(2):
            pair.step(_grads(numel, 2, "f32", 20 + t))
            pair.compare(f"step {t}")
            _check(pair, reps, rep_dtype, f"misaligned step {t}")
    finally:
        pair.close()


def test_half_replicas_round_large_tiny_and_tied_weights():
    """Weights chosen so that the fp16 replicas hit overflow, subnormals and exact ties."""
    vals = np.array([65519.0, 65520.0, 70000.0, -70000.0, 2.0 ** -25, 1.5 * 2.0 ** -24, 2.0 ** -24, 3e-8, -3e-8,
                     1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2049.0, 2051.0, 0.1, -0.1, 0.0], dtype=F)
    pair = Pair([vals.size], 1, "f32", 4096, lr=0.0, momentum=0.0, wd=0.0, rescale=1.0)
    try:
        pair.set_weights([vals])
        reps = _replicas([vals.size], 2, "f16")
        pair.gpu.set_broadcast(0, reps[0], "f16")
        pair.step([[np.zeros(vals.size, dtype=F)]])             # lr = 0: w' = w
        pair.compare("rounding")
        _check(pair, reps, "f16", "rounding")
        with np.errstate(over="ignore"):
            assert np.array_equal(reps[0][0].cpu().numpy().view(np.uint16), vals.astype(np.float16).view(np.uint16))
    finally:
        pair.close()


def test_only_some_keys_have_replicas_and_they_can_be_removed():
    import torch
    numel = [3000, 3000, 3000]
    pair = Pair(numel, 2, "f32", 1 << 20, lr=0.1, momentum=0.0, wd=0.0)
    try:
        reps = _replicas(numel, 2, "f32")
        pair.gpu.set_broadcast(1, reps[1], "f32")
        pair.step(_grads(numel, 2, "f32", 30))
        assert torch.all(reps[0][0] == 7.0) and torch.all(reps[2][1] == 7.0)
        assert same_bits_or_both_nan(reps[1][0].cpu().numpy(), pair.cpu.w[1])
        # a different replica count or dtype on the same store is refused
        with pytest.raises(pair.kv.KVError) as e:
            pair.gpu.set_broadcast(0, reps[0][:1], "f32")
        assert e.value.status == -3
        with pytest.raises(pair.kv.KVError):
            pair.gpu.set_broadcast(0, _replicas([3000], 2, "f16")[0], "f16")
        with pytest.raises(pair.kv.KVError) as e:
            pair.gpu.set_broadcast(0, [reps[0][0].data_ptr() + 2, reps[0][1].data_ptr()], "f32")
        assert e.value.status == -4
        pair.gpu.set_broadcast(1, [], "f32")                     # remove
        before = reps[1][0].clone()
        pair.step(_grads(numel, 2, "f32", 31))
        assert torch.equal(reps[1][0], before)
        pair.compare("after removal")
    finally:
        pair.close()


@pytest.mark.timeout(300)
def test_resnet50_full_size_with_half_replicas():
    """ResNet-50-shaped set, W = 32 fp16 gradients, one fp16 weight copy per key (what a
    mixed-precision forward pass reads), at full size."""
    import torch
    cfg = wl.get_config(4)
    pair = Pair(cfg.numel, cfg.W, "f16", cfg.bucket_bytes, lr=cfg.lr, momentum=cfg.momentum, wd=cfg.wd, keep_sum=False)
    try:
        pair.set_weights(wl.make_weights(cfg, 16))
        reps = [[torch.empty(n, dtype=torch.float16, device="cuda")] for n in cfg.numel]
        for k in range(len(cfg.numel)):
            pair.gpu.set_broadcast(k, reps[k], "f16")
        pair.step(wl.make_step_gradients(cfg, 0, 16), oracle_threads=8)
        pair.compare("cfg4 + f16 replica")
        _check(pair, reps, "f16", "cfg4")
    finally:
        pair.close()


def test_broadcast_of_current_weights_skips_keys_without_replicas_and_refuses_pending_keys():
    import torch
    numel = [300, 5000, 64]
    pair = Pair(numel, 2, "f32", 1 << 20, lr=0.1, momentum=0.9, wd=1e-4)
    try:
        pair.set_weights([_rng(3, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        pair.gpu.broadcast_weights()                       # no replicas at all: nothing to do
        reps = _replicas(numel, 2, "f16")
        pair.gpu.set_broadcast(1, reps[1], "f16")          # only key 1
        pair.gpu.broadcast_weights()
        pair.gpu.wait()
        ref = orc.round_to_half(pair.cpu.w[1])
        for t in reps[1]:
            assert np.array_equal(t.cpu().numpy().view(np.uint16), ref.view(np.uint16))
        for k in (0, 2):
            for t in reps[k]:
                assert torch.all(t == 7.0)                 # untouched
        dev = pair.upload(_grads(numel, 2, "f32", 30))
        pair.gpu.push(1, dev[1])                           # keys 0..2 share a bucket: key 1 now waits for the others
        with pytest.raises(pair.kv.KVError) as e:
            pair.gpu.broadcast_weights(1)
        assert e.value.status == -3
        with pytest.raises(pair.kv.KVError):
            pair.gpu.broadcast_weights(3)
        pair.gpu.push(0, dev[0])
        pair.gpu.push(2, dev[2])
        pair.gpu.wait()
    finally:
        pair.close()
