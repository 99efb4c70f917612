"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle,
element by element on the same seeded inputs.

Bar: bit-exact raw sums, weights and momentum (same operation order on both
sides, IEEE binary32, one rounding per operation).  This is stricter than the
1e-6 (fp32) / 1e-3 (fp16 gradients) relative tolerances the target allows, so
those are not used.  NaN payloads are the one exception (both sides NaN).
"""
from __future__ import annotations

import numpy as np
import pytest

import workloads as wl
from oracle import kv_oracle as orc
from tests.gpu_harness import Pair, run_config, same_bits_or_both_nan, to_device
from tests.helpers import load_hand_cases

pytestmark = pytest.mark.gpu
F = np.float32


def _rng(*seed):
    return np.random.Generator(np.random.SFC64(list(seed)))


def _grads(numel, W, dtype, seed, scale=0.01):
    out = []
    for k, n in enumerate(numel):
        gk = [(_rng(seed, k, r).standard_normal(n, dtype=F) * F(scale)).astype(F) for r in range(W)]
        if dtype == "f16":
            gk = [g.astype(np.float16) for g in gk]
        out.append(gk)
    return out


# Lengths that straddle the vector width, the wavefront, the workgroup and the
# tile sizes (256 * lane_elems * unroll elements: 256 ... 4096), plus empty keys.
RAGGED = [0, 1, 2, 3, 4, 5, 7, 8, 9, 63, 64, 65, 255, 256, 257, 1023, 1024, 1025, 2047, 2048, 2049,
          4095, 4096, 4097, 8191, 8192, 8193, 0, 12289, 20000]


# ------------------------------------------------------------------ benchmark configurations
@pytest.mark.parametrize("order", [orc.SEQUENTIAL, orc.PAIRWISE])
@pytest.mark.parametrize("mode", ["list", "each"])
def test_config1_mlp(order, mode):
    run_config(wl.get_config(1), 3, order=order, mode=mode)


@pytest.mark.parametrize("order", [orc.SEQUENTIAL, orc.PAIRWISE])
@pytest.mark.parametrize("mode", ["list", "each"])
def test_config2_resnet20(order, mode):
    run_config(wl.get_config(2), 3, order=order, mode=mode)


@pytest.mark.timeout(300)
@pytest.mark.parametrize("order", [orc.SEQUENTIAL, orc.PAIRWISE])
def test_config3_resnet50_full_size(order):
    """Full 25.6M-parameter key set, W = 8, in the launch configuration the
    benchmark times (list push, default tuning, raw sums not stored)."""
    run_config(wl.get_config(3), 3, order=order, keep_sum=(order == orc.PAIRWISE), gen_threads=16, oracle_threads=8)


@pytest.mark.timeout(300)
def test_config4_resnet50_half_gradients_full_size():
    run_config(wl.get_config(4), 2, gen_threads=16, oracle_threads=8)


@pytest.mark.timeout(600)
def test_config5_vgg16_full_size():
    """138M parameters, W = 16: one freshly generated step and a second one that
    reuses those gradients with the ranks rotated (so that m != 0 is covered
    without another 2.2e9 normal draws)."""
    run_config(wl.get_config(5), 2, keep_sum=False, gen_threads=16, oracle_threads=8, rotate_after_first=True)


@pytest.mark.timeout(300)
def test_config6_inception_bn_with_the_papers_learning_rate_scaling():
    """The paper's other ImageNet model; the learning rate is changed between steps with
    kv_set_lr along the linear scaling the paper describes (0.1 by default, 1.0 at 256 GPUs)."""
    cfg = wl.get_config(6)
    pair = Pair(cfg.numel, cfg.W, cfg.grad_dtype, cfg.bucket_bytes, lr=wl.scaled_lr(8), momentum=cfg.momentum, wd=cfg.wd)
    try:
        pair.set_weights(wl.make_weights(cfg, 16))
        for t, gpus in enumerate((8, 64, 256)):
            lr = wl.scaled_lr(gpus)
            pair.gpu.set_lr(lr)
            pair.cpu.lr = lr
            pair.step(wl.make_step_gradients(cfg, t, 16), oracle_threads=8)
            pair.compare(f"inception-bn step {t} lr {lr}")
    finally:
        pair.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("dtype,numel,W", [("f32", (1 << 30) + 517, 1), ("f16", (1 << 31) + 1029, 2)])
def test_one_key_beyond_four_gigabytes(dtype, numel, W):
    """Maximum sizes: element and byte offsets of a single key pass 2^31 and 2^32.
    Values repeat a 16M-element seeded block (cheap to generate, same on both sides)."""
    block = 1 << 24
    reps = numel // block + 1

    def tiled(seed, scale, dt):
        b = (_rng(seed).standard_normal(block, dtype=F) * F(scale)).astype(dt)
        return np.tile(b, reps)[:numel]

    pair = Pair([64, numel, 5], W, dtype, 1 << 20, lr=0.1, momentum=0.9, wd=1e-4, keep_sum=False)
    try:
        gdt = np.float32 if dtype == "f32" else np.float16
        small = lambda n, seed: [(_rng(seed, r).standard_normal(n, dtype=F) * F(0.01)).astype(gdt) for r in range(W)]
        grads = [small(64, 71), [tiled(72 + r, 0.01, gdt) for r in range(W)], small(5, 73)]
        pair.set_weights([_rng(74).standard_normal(64, dtype=F), tiled(75, 1.0, F), _rng(76).standard_normal(5, dtype=F)])
        dev = pair.step(grads, oracle_threads=16)
        pair.step(grads, dev=dev, oracle_threads=16)                   # second step: m != 0
        pair.compare(f"{numel} elements of {dtype}")
    finally:
        pair.close()


# ------------------------------------------------------------------ ragged sizes, every W path
@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("W", [1, 2, 3, 4, 5, 7, 8, 9, 13, 15, 16, 17, 24, 32, 33, 40, 64, 100])
@pytest.mark.parametrize("order", [orc.SEQUENTIAL, orc.PAIRWISE])
def test_ragged_keys_all_rank_counts(dtype, W, order):
    pair = Pair(RAGGED, W, dtype, 16 << 10, lr=0.1, momentum=0.9, wd=1e-4, order=order)
    try:
        pair.set_weights([_rng(1, k).standard_normal(n, dtype=F) for k, n in enumerate(RAGGED)])
        for t in range(2):
            pair.step(_grads(RAGGED, W, dtype, 100 + t))
            pair.compare(f"W={W} {dtype} order={order} step {t}")
    finally:
        pair.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("lane_elems", [1, 2, 4])
@pytest.mark.parametrize("W", [3, 5, 9, 12, 15, 17, 20, 31, 33, 36, 40, 47, 63, 64, 65, 72, 100])
def test_run_time_rank_counts_at_every_lane_width(dtype, lane_elems, W):
    """The kernel for a W known only at run time folds whole large batches, a half batch, whole small batches and
    a tail of 4 + 2 + 1 ranks; the batch sizes depend on the size of a lane's vector (2 to 16 bytes).  Every
    boundary of that scheme, in both fold orders (pairwise on the odd counts)."""
    order = orc.PAIRWISE if W % 2 else orc.SEQUENTIAL
    numel = [1, 255, 1024 + 7, 6000]
    pair = Pair(numel, W, dtype, 16 << 10, lr=0.1, momentum=0.9, wd=1e-4, order=order, lane_elems=lane_elems)
    try:
        pair.set_weights([_rng(9, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        for t in range(2):
            pair.step(_grads(numel, W, dtype, 9000 + 7 * W + t))
            pair.compare(f"W={W} {dtype} lane={lane_elems} order={order} step {t}")
    finally:
        pair.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("W", [2, 4, 8, 16, 32])
@pytest.mark.parametrize("order", [orc.SEQUENTIAL, orc.PAIRWISE])
def test_run_time_w_kernel_at_the_rank_counts_that_have_a_kernel_of_their_own(dtype, W, order):
    """tuning.run_time_w sends W = 2 ... 32 through the kernel that takes W at run time: same bits as the oracle,
    hence as the kernels built for those W."""
    pair = Pair(RAGGED, W, dtype, 16 << 10, lr=0.1, momentum=0.9, wd=1e-4, order=order, run_time_w=1)
    try:
        assert pair.gpu.get_tuning()[0]["run_time_w"] == 1
        pair.set_weights([_rng(1, k).standard_normal(n, dtype=F) for k, n in enumerate(RAGGED)])
        for t in range(2):
            pair.step(_grads(RAGGED, W, dtype, 100 + t))
            pair.compare(f"run-time-W kernel W={W} {dtype} order={order} step {t}")
    finally:
        pair.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("lane_elems,unroll", [(4, 1), (4, 2), (4, 4), (2, 1), (2, 2), (1, 1), (1, 2), (1, 4)])
@pytest.mark.parametrize("tuning", [dict(), dict(workgroups_per_cu=1), dict(xcd_remap=0), dict(nontemporal=0), dict(nontemporal=1), dict(nontemporal=5), dict(nontemporal=9), dict(nontemporal=13),
                                    dict(workgroups_per_cu=2, xcd_remap=1), dict(workgroups_per_cu=3, xcd_remap=0), dict(xcd_remap=1),
                                    dict(xcd_remap=7), dict(xcd_remap=3, workgroups_per_cu=1), dict(xcd_remap=4096),
                                    dict(resident_workgroups=3), dict(resident_workgroups=5, xcd_remap=16)])
def test_tuning_never_changes_a_bit(dtype, lane_elems, unroll, tuning):
    numel = RAGGED + [70001]
    pair = Pair(numel, 8, dtype, 64 << 10, lr=0.1, momentum=0.9, wd=1e-4, unroll=unroll, lane_elems=lane_elems, **tuning)
    try:
        pair.set_weights([_rng(2, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        for t in range(2):
            pair.step(_grads(numel, 8, dtype, 200 + t))
            pair.compare(f"lane_elems={lane_elems} unroll={unroll} {tuning} step {t}")
    finally:
        pair.close()


@pytest.mark.parametrize("dtype,W,lazy", [("f32", 8, False), ("f16", 32, False), ("f32", 3, True)])
def test_store_that_tunes_itself_never_changes_a_bit(dtype, W, lazy):
    """KV_FLAG_AUTOTUNE: the first launches each try another launch shape; every step still matches the oracle, and
    the store settles on one of the shapes it tried."""
    numel = RAGGED + [70001, 300000]
    pair = Pair(numel, W, dtype, 64 << 10, lr=0.1, momentum=0.9, wd=1e-4, autotune=True, lazy=lazy, keep_sum=False)
    try:
        pair.set_weights([_rng(4, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        sets = [_grads(numel, W, dtype, 400 + j) for j in range(2)]
        dev = [pair.upload(g) for g in sets]
        seen, done = set(), False
        for t in range(48):
            tuning, done = pair.gpu.get_tuning()
            seen.add((tuning["lane_elems"], tuning["resident_workgroups"], tuning["xcd_remap"]))
            pair.step(sets[t % 2], dev=dev[t % 2], mode="each" if lazy else "list")
            if t % 6 == 0 or t > 40:
                pair.compare(f"self-tuning step {t}")
        pair.compare("after tuning")
        tuning, done = pair.gpu.get_tuning()
        assert done and len(seen) >= 12                      # 12 lane x cap candidates, then XCD blocks
        assert tuning["lane_elems"] in (1, 2, 4) and tuning["unroll"] == 1 and tuning["resident_workgroups"] in (4, 5, 6, 8)
        assert (tuning["lane_elems"], tuning["resident_workgroups"], tuning["xcd_remap"]) in seen
    finally:
        pair.close()


@pytest.mark.parametrize("seed", range(12))
def test_random_tuning_on_random_key_sets(seed):
    """Random launch shapes, cache policies, XCD blocks and occupancy caps on random ragged key sets, rank counts with
    and without a kernel of their own, both dtypes and both orders: never a bit of difference."""
    r = _rng(900, seed)
    K = int(r.integers(1, 12))
    numel = [int(x) for x in r.choice([0, 1, 3, 17, 255, 256, 257, 1000, 1024, 4097, 10000, 33333, 70001], size=K)]
    W = int(r.choice([1, 2, 3, 4, 5, 8, 13, 16, 32, 40]))
    dtype = "f16" if r.integers(2) else "f32"
    lane, unroll = [(4, 1), (4, 2), (4, 4), (2, 1), (2, 2), (1, 1), (1, 2), (1, 4)][int(r.integers(8))]
    tuning = dict(lane_elems=lane, unroll=unroll, nontemporal=int(r.choice([0, 1, 5, 9, 13])),
                  xcd_remap=int(r.choice([0, 1, 2, 5, 16, 64, 1000])), resident_workgroups=int(r.choice([0, 3, 4, 6, 8])),
                  workgroups_per_cu=int(r.choice([0, 0, 1, 2])))
    pair = Pair(numel, W, dtype, int(r.choice([64, 4096, 1 << 16, 1 << 22])), lr=0.05, momentum=0.8, wd=1e-3,
                order=int(r.integers(2)), **tuning)
    try:
        pair.set_weights([_rng(901, seed, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        for t in range(2):
            pair.step(_grads(numel, W, dtype, 1000 + 10 * seed + t), mode="each" if t else "list")
            pair.compare(f"seed {seed} W={W} {dtype} {numel} {tuning} step {t}")
    finally:
        pair.close()


@pytest.mark.parametrize("lane", [1, 2, 4])
@pytest.mark.parametrize("W,dtype", [(4, "f32"), (5, "f32"), (8, "f16"), (40, "f16"), (33, "f32")])
def test_one_misaligned_buffer_among_aligned_ones(W, dtype, lane):
    """The kernel gets the OR of all gradient pointers of a launch and skips its per-key alignment check when
    that is aligned for its lane width.  Here a single rank of a single key starts one element into its
    allocation: that key must take the single-element path, every other key the vector path, and both must
    give the oracle's bits; in the second step no buffer is misaligned."""
    numel = [700, 2048, 4096 + 3, 12289, 64]
    pair = Pair(numel, W, dtype, 8 << 10, lr=0.1, momentum=0.9, wd=1e-4, lane_elems=lane)
    try:
        pair.set_weights([_rng(5, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        for t in range(2):
            grads = _grads(numel, W, dtype, 7000 + 10 * W + t)
            dev = [[to_device(g, 1 if (t == 0 and k == 3 and r == W - 1) else 0) for r, g in enumerate(gk)]
                   for k, gk in enumerate(grads)]
            pair.step(grads, dev=dev)
            pair.compare(f"W={W} {dtype} lane={lane} step {t}")
    finally:
        pair.close()


@pytest.mark.parametrize("W,dtype", [(8, "f32"), (16, "f32"), (16, "f16"), (32, "f16"), (40, "f16"), (33, "f32")])
@pytest.mark.parametrize("mode", ["list", "each"])
def test_views_off_the_line_grid_take_the_wide_shape_and_the_same_bits(W, dtype, mode):
    """Gradient views that start 32 bytes off a 128-byte line (but on a 4-element vector): a store whose default
    is one element per lane (or two, with 8 and more ranks) launches them with four.  Step 0: all keys off the grid (wide launches); step 1: only a
    small key off the grid (default shape); step 2: one buffer 4 bytes off (no 4-element vectors: default shape)."""
    numel = [4096, 300, 40000 + 12, 1024, 70000]
    isz = 4 if dtype == "f32" else 2
    pair = Pair(numel, W, dtype, 64 << 10, lr=0.1, momentum=0.9, wd=1e-4)
    try:
        assert pair.gpu.get_tuning()[0]["lane_elems"] == (2 if W == 16 else 1)
        pair.set_weights([_rng(6, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        wide_before = pair.gpu.wide_launches()
        for t in range(3):
            grads = _grads(numel, W, dtype, 8000 + 10 * W + t)
            def off(k, r):
                if t == 0:
                    return 32 // isz
                if t == 1:
                    return 32 // isz if k == 1 else 0
                return 1 if (k == 4 and r == 0) else 32 // isz
            dev = [[to_device(g, off(k, r)) for r, g in enumerate(gk)] for k, gk in enumerate(grads)]
            pair.step(grads, dev=dev, mode=mode)
            pair.compare(f"W={W} {dtype} {mode} step {t}")
            wide = pair.gpu.wide_launches() - wide_before
            if t == 0:
                assert wide >= 1, "buffers off the line grid did not take the wide shape"
                wide_after_first = wide
            else:
                assert wide == wide_after_first or mode == "each", (t, wide, wide_after_first)
    finally:
        pair.close()


def test_a_fixed_lane_width_is_never_overridden():
    numel = [4096, 70000]
    pair = Pair(numel, 8, "f32", 64 << 10, lr=0.1, momentum=0.9, wd=1e-4, lane_elems=1)
    try:
        pair.set_weights([_rng(7, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        grads = _grads(numel, 8, "f32", 8100)
        pair.step(grads, dev=[[to_device(g, 8) for g in gk] for gk in grads])
        pair.compare("fixed lane width")
        assert pair.gpu.wide_launches() == 0
    finally:
        pair.close()


@pytest.mark.parametrize("dtype,misalign", [("f32", 1), ("f32", 2), ("f32", 3), ("f16", 1), ("f16", 2), ("f16", 4), ("f16", 7)])
def test_gradient_buffers_not_16_byte_aligned(dtype, misalign):
    """Views into a flat buffer: aligned to the element only, so the single-element path runs."""
    numel = [5, 1000, 4096, 9001]
    pair = Pair(numel, 4, dtype, 8 << 10, lr=0.1, momentum=0.9, wd=1e-4)
    try:
        pair.set_weights([_rng(3, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        for t in range(2):
            pair.step(_grads(numel, 4, dtype, 300 + t), misalign=misalign)
            pair.compare(f"misalign={misalign} step {t}")
    finally:
        pair.close()


@pytest.mark.parametrize("bucket", [1, 4096, 1 << 40])
def test_bucket_size_never_changes_a_bit(bucket):
    numel = [10, 3000, 64, 1024, 5000, 7, 256]
    pair = Pair(numel, 8, "f32", bucket, lr=0.1, momentum=0.9, wd=1e-4)
    try:
        pair.set_weights([_rng(4, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        for t in range(2):
            pair.step(_grads(numel, 8, "f32", 400 + t))
            pair.compare(f"bucket={bucket} step {t}")
    finally:
        pair.close()


# ------------------------------------------------------------------ worked examples and special values
@pytest.mark.parametrize("case", load_hand_cases(), ids=lambda c: c["name"])
def test_hand_computed_cases_on_gpu(case):
    dt = np.float32 if case["dtype"] == "f32" else np.float16
    g = [np.array(r, dtype=dt) for r in case["g"]]
    n = len(case["w"])
    pair = Pair([n], len(g), case["dtype"], 4096, lr=case["lr"], momentum=case["momentum"], wd=case["wd"],
                rescale=case["rescale"], order=case["order"])
    try:
        pair.set_weights([np.array(case["w"], dtype=F)])
        pair.set_momentum([np.array(case["m"], dtype=F)])
        pair.step([g])
        assert np.array_equal(pair.fetch("s", 0), np.array(case["expect_s"], dtype=F))
        assert np.array_equal(pair.fetch("m", 0), np.array(case["expect_m"], dtype=F))
        assert np.array_equal(pair.fetch("w", 0), np.array(case["expect_w"], dtype=F))
    finally:
        pair.close()


@pytest.mark.parametrize("W", [1, 2, 3, 4, 8])
def test_kvstore_snippet_on_gpu(W):
    """KVStore API section: every worker pushes ones((2,3)); pull returns W * ones."""
    pair = Pair([6], W, "f32", 4096, lr=0.1, momentum=0.0, wd=0.0)
    try:
        pair.step([[np.ones(6, dtype=F) for _ in range(W)]])
        assert np.array_equal(pair.fetch("s", 0), np.full(6, W, dtype=F))
    finally:
        pair.close()


def test_every_half_bit_pattern_widens_exactly():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    pair = Pair([65536], 1, "f16", 1 << 20, lr=0.0, momentum=0.0, wd=0.0, rescale=1.0)
    try:
        pair.step([[h]])
        pair.compare("all halves")
        with np.errstate(invalid="ignore"):
            ref = h.astype(np.float32)
        assert same_bits_or_both_nan(pair.fetch("s", 0), ref)
    finally:
        pair.close()


def test_subnormals_signed_zeros_inf_nan():
    tiny = np.array([1, 2, 0x007FFFFF, 0x80000001], dtype=np.uint32).view(F)
    special = np.array([-0.0, 0.0, np.inf, -np.inf, np.nan, 1e-45, -1e-45, 3e38], dtype=F)
    g0 = np.concatenate([tiny, special, np.full(4, -0.0, dtype=F)])
    g1 = np.concatenate([tiny, special[::-1], np.full(4, -0.0, dtype=F)])
    n = g0.size
    for order in (orc.SEQUENTIAL, orc.PAIRWISE):
        pair = Pair([n], 2, "f32", 4096, lr=1.0, momentum=0.5, wd=0.0, rescale=1.0, order=order)
        try:
            pair.set_weights([np.linspace(-1, 1, n).astype(F) * F(1e-40)])
            pair.set_momentum([np.full(n, 1e-42, dtype=F)])
            with np.errstate(all="ignore"):
                pair.step([[g0, g1]])
            pair.compare("special values")
            s = pair.fetch("s", 0)
            assert np.all(s[-4:].view(np.uint32) == 0x80000000)       # -0 + -0 stays -0
            assert s.view(np.uint32)[0] == 2                          # subnormal sum is kept
        finally:
            pair.close()


def test_operations_are_not_fused_on_gpu():
    a = F(1 + 2.0 ** -12)
    pair = Pair([1], 1, "f32", 4096, lr=1.0, momentum=float(a), wd=0.0, rescale=1.0)
    try:
        pair.set_momentum([np.array([a], dtype=F)])
        pair.step([[np.array([1 + 2.0 ** -11], dtype=F)]])
        assert pair.fetch("m", 0)[0] == 0.0                          # a fused multiply-add would leave 2^-24
        pair.compare("no fma")
    finally:
        pair.close()


# ------------------------------------------------------------------ ordering, chain, pulls
def test_push_order_changes_nothing_and_launches_ascend():
    cfg = wl.get_config(2)
    K = len(cfg.keys)
    weights = wl.make_weights(cfg)
    grads = [wl.make_step_gradients(cfg, t) for t in range(2)]
    orders = [list(range(K)), list(range(K))[::-1], [int(x) for x in _rng(5).permutation(K)]]
    results = []
    for o in orders:
        pair = Pair(cfg.numel, cfg.W, "f32", cfg.bucket_bytes, lr=cfg.lr, momentum=cfg.momentum, wd=cfg.wd)
        try:
            pair.set_weights(weights)
            for t in range(2):
                pair.step(grads[t], mode="each", order=o)
            pair.compare(f"order {o[:4]}...")
            total, log = pair.gpu.launch_log()
            U = pair.gpu.plan.num_units
            covered = []
            for first, n in log:
                covered += list(range(first, first + n))
            assert covered == list(range(U)) * 2, "every unit once per iteration, ascending"
            results.append([pair.fetch("w", k) for k in range(K)])
        finally:
            pair.close()
    for r in results[1:]:
        for a, b in zip(r, results[0]):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_native_repeat_of_a_list_push_is_that_many_steps():
    """kv_push_list_repeat (a timing helper): n calls of kv_push_list with the same buffers, from native code."""
    numel = [100, 5000, 0, 1025]
    pair = Pair(numel, 4, "f32", 8 << 10, lr=0.1, momentum=0.9, wd=1e-4)
    try:
        pair.set_weights([_rng(11, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        grads = _grads(numel, 4, "f32", 1100)
        dev = pair.upload(grads)
        before = pair.gpu.launch_log(0)[0]
        pair.gpu.push_list_repeat(pair.gpu.make_push_list(list(range(len(numel))), dev), 3)
        pair.gpu.wait()
        assert pair.gpu.launch_log(0)[0] - before == 3
        for _ in range(3):
            pair.cpu.step(grads)
        pair.compare("three native repeats")
        with pytest.raises(Exception):
            pair.gpu.push_list_repeat(pair.gpu.make_push_list([0], [dev[0]]), 0)
    finally:
        pair.close()


def test_list_push_is_one_launch_per_iteration():
    cfg = wl.get_config(2)
    pair = Pair(cfg.numel, cfg.W, "f32", cfg.bucket_bytes, lr=cfg.lr, momentum=cfg.momentum, wd=cfg.wd)
    try:
        g = wl.make_step_gradients(cfg, 0)
        dev = pair.step(g)
        pair.step(g, dev=dev)
        total, log = pair.gpu.launch_log()
        assert total == 2 and log == [(0, pair.gpu.plan.num_units)] * 2
    finally:
        pair.close()


def test_alternating_gradient_buffers_use_the_right_pointers():
    """The device pointer tables are cached; cycling through more buffer sets than
    there are cached tables must still read the set that was pushed."""
    numel = [100, 5000, 64, 3000]
    W = 2
    pair = Pair(numel, W, "f32", 4096, lr=0.1, momentum=0.9, wd=1e-4)
    try:
        sets = [_grads(numel, W, "f32", 500 + i) for i in range(6)]
        devs = [pair.upload(s) for s in sets]
        seq = [0, 1, 0, 1, 2, 3, 4, 5, 0, 5, 2, 2, 1]
        for i, which in enumerate(seq):
            mode = "each" if i % 3 == 2 else "list"
            pair.step(sets[which], dev=devs[which], mode=mode)
            pair.compare(f"alternation step {i} set {which}")
    finally:
        pair.close()


def test_pull_before_the_bucket_is_complete_is_deferred():
    import torch
    numel = [8, 8, 8]                                   # one bucket
    pair = Pair(numel, 2, "f32", 4096, lr=0.5, momentum=0.0, wd=0.0)
    try:
        g = _grads(numel, 2, "f32", 600, scale=1.0)
        dev = pair.upload(g)
        out = torch.full((8,), 7.0, device="cuda")
        pair.gpu.push(0, dev[0])
        pair.gpu.pull(0, out)                           # unit not launched yet: queued
        assert pair.gpu.wait_status(0) == -5            # KV_ERR_INCOMPLETE, does not block
        assert pair.gpu.wait_status(-1) == -5
        assert torch.all(out == 7.0)
        pair.gpu.push(2, dev[2])
        pair.gpu.push(1, dev[1])                        # completes the bucket: launch, then the queued pull
        pair.gpu.wait()
        pair.cpu.step(g)
        assert np.array_equal(out.cpu().numpy(), pair.cpu.w[0])
        pair.compare("deferred pull")
    finally:
        pair.close()


@pytest.mark.parametrize("schedule", [None, (1, 1, 0), (2, 3, 0)], ids=["chained", "funnel", "concurrent"])
def test_list_pull_gathers_whole_keys(schedule):
    import torch
    numel = [0, 1, 5, 64, 1023, 1025, 4096, 4099, 0, 20000, 7]
    pair = Pair(numel, 2, "f32", 8192, lr=0.1, momentum=0.9, wd=1e-4, schedule=schedule)
    try:
        pair.set_weights([_rng(9, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        pair.step(_grads(numel, 2, "f32", 650))
        K = len(numel)
        for keys, mis in ((list(range(K)), 0), ([9, 2, 3, 6], 0), ([1, 2, 4, 5, 10], 1), ([3, 3], 0)):
            bufs = [torch.full((numel[k] + 8,), 7.0, device="cuda") for k in keys]
            outs = [b[mis:mis + numel[k]] for b, k in zip(bufs, keys)]
            pair.gpu.pull_list(keys, outs)
            pair.gpu.wait()
            for k, o, b in zip(keys, outs, bufs):
                assert np.array_equal(o.cpu().numpy().view(np.uint32), pair.cpu.w[k].view(np.uint32)), (keys, k)
                assert torch.all(b[mis + numel[k]:] == 7.0) and torch.all(b[:mis] == 7.0)   # nothing outside the key
        # a listed key that still waits for its launch is served after that launch
        if schedule is None:
            g = _grads(numel, 2, "f32", 651)
            dev = pair.upload(g)
            outs = [torch.zeros(numel[k], device="cuda") for k in range(K)]
            pair.gpu.push(3, dev[3])
            pair.gpu.pull_list(list(range(K)), outs)
            for k in range(K):
                if k != 3:
                    pair.gpu.push(k, dev[k])
            pair.gpu.wait()
            pair.cpu.step(g)
            assert np.array_equal(outs[3].cpu().numpy(), pair.cpu.w[3])
        with pytest.raises(pair.kv.KVError):
            pair.gpu.pull_list([0, 99], [torch.zeros(1, device="cuda")] * 2)
    finally:
        pair.close()


def test_large_key_waits_for_lower_units():
    """Chain order: a ready unit still waits for every lower unit."""
    numel = [16, 4096, 16]                               # bucket {0, 2} is unit 0, key 1 (large) is unit 1
    pair = Pair(numel, 2, "f32", 1024, lr=0.1, momentum=0.0, wd=0.0)
    try:
        assert pair.gpu.plan.units() == [([0, 2], False), ([1], True)]
        g = _grads(numel, 2, "f32", 700)
        dev = pair.upload(g)
        pair.gpu.push(1, dev[1])
        assert pair.gpu.launch_log()[0] == 0
        pair.gpu.push(0, dev[0])
        assert pair.gpu.launch_log()[0] == 0
        pair.gpu.push(2, dev[2])
        total, log = pair.gpu.launch_log()
        assert total == 1 and log == [(0, 2)]
        pair.gpu.wait()
        pair.cpu.step(g)
        pair.compare("chain")
    finally:
        pair.close()


def test_errors_leave_the_store_usable():
    import torch
    kv = pytest.importorskip("paper_1802_06949_amd")
    numel = [16, 16]
    pair = Pair(numel, 2, "f32", 4096, lr=0.1, momentum=0.0, wd=0.0, keep_sum=False)
    try:
        g = _grads(numel, 2, "f32", 800)
        dev = pair.upload(g)
        ptrs0 = [t.data_ptr() for t in dev[0]]
        assert pair.gpu.push_raw(5, ptrs0) == -2                        # KV_ERR_KEY
        assert pair.gpu.push_raw(0, [ptrs0[0] + 2, ptrs0[1]]) == -4     # KV_ERR_ALIGN
        assert pair.gpu.push_raw(0, [0, ptrs0[1]]) == -1                # KV_ERR_ARG
        assert pair.gpu.push_raw(0, ptrs0) == 0
        assert pair.gpu.push_raw(0, ptrs0) == -3                        # KV_ERR_STATE: second push
        assert "twice" in pair.gpu.last_error()
        with pytest.raises(kv.KVError):
            pair.gpu.pull_grad(0, torch.empty(16, device="cuda"))       # store has no raw-sum arena
        with pytest.raises(kv.KVError):
            pair.gpu.push_list(pair.gpu.make_push_list([1, 1], [dev[1], dev[1]]))
        pair.gpu.push(1, dev[1])
        pair.gpu.wait()
        pair.cpu.step(g)
        pair.compare("after errors")
    finally:
        pair.close()


def test_learning_rate_change_and_checkpoint_round_trip():
    numel = [100, 3000, 17]
    W = 4
    a = Pair(numel, W, "f32", 4096, lr=0.1, momentum=0.9, wd=1e-4)
    b = None
    try:
        a.set_weights([_rng(6, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        a.step(_grads(numel, W, "f32", 900))
        a.gpu.set_lr(0.01); a.cpu.lr = 0.01
        a.step(_grads(numel, W, "f32", 901))
        a.compare("after lr change")
        # save, restore into a fresh store, continue: bit-identical to continuing in place
        w = [a.fetch("w", k) for k in range(len(numel))]
        m = [a.fetch("m", k) for k in range(len(numel))]
        b = Pair(numel, W, "f32", 4096, lr=0.01, momentum=0.9, wd=1e-4)
        b.set_weights(w); b.set_momentum(m)
        g = _grads(numel, W, "f32", 902)
        a.step(g); b.step(g)
        b.compare("restored")
        for k in range(len(numel)):
            assert np.array_equal(a.fetch("w", k).view(np.uint32), b.fetch("w", k).view(np.uint32))
    finally:
        a.close()
        if b is not None:
            b.close()


def test_optimizer_parameters_can_change_between_steps():
    numel = [100, 3000, 17]
    W = 4
    pair = Pair(numel, W, "f32", 4096, lr=0.1, momentum=0.0, wd=0.0)
    try:
        pair.set_weights([_rng(14, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        assert pair.gpu.get_sgd_params()["rescale"] == 0.25
        for t, (lr, mu, wd, rs, order) in enumerate([(0.1, 0.0, 0.0, 0.0, 0), (0.05, 0.9, 1e-3, 0.0, 1),
                                                      (0.2, 0.5, 0.0, 1.0, 0), (0.0, 0.9, 1e-2, 0.125, 1)]):
            pair.gpu.set_sgd_params(lr=lr, momentum=mu, wd=wd, rescale=rs, reduce_order=order)
            pair.cpu.lr, pair.cpu.momentum, pair.cpu.wd, pair.cpu.order = lr, mu, wd, order
            pair.cpu.rescale = rs if rs > 0 else float(F(1) / F(W))
            got = pair.gpu.get_sgd_params()
            assert got["reduce_order"] == order and got["rescale"] == F(pair.cpu.rescale)
            pair.step(_grads(numel, W, "f32", 1200 + t))
            pair.compare(f"parameters {t}")
        with pytest.raises(pair.kv.KVError):
            pair.gpu.set_sgd_params(lr=0.1, momentum=0.0, wd=0.0, reduce_order=5)
    finally:
        pair.close()


def test_zero_copy_weights_pointer_and_timing():
    import ctypes
    import torch
    numel = [64, 5000]
    pair = Pair(numel, 2, "f32", 4096, lr=0.1, momentum=0.0, wd=0.0)
    try:
        g = _grads(numel, 2, "f32", 1000)
        pair.gpu.timing_begin()
        pair.step(g)
        pair.gpu.timing_mark()
        dev = pair.step(g)
        pair.step(g, dev=dev)
        pair.gpu.timing_mark()
        ms, launches = pair.gpu.timing_end()
        iv = pair.gpu.timing_intervals()
        assert launches == 3 and ms > 0 and len(iv) == 2 and all(x > 0 for x in iv) and sum(iv) <= ms * 1.001
        ptr = pair.gpu.weights_ptr(1)
        assert ptr % 16 == 0
        out = torch.empty(5000, device="cuda")
        pair.kv.copy_bytes(out, type("P", (), {"data_ptr": lambda self: ptr})(), 5000 * 4)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), pair.cpu.w[1])
    finally:
        pair.close()


@pytest.mark.parametrize("seed", range(6))
def test_random_sessions_of_pushes_and_pulls(seed):
    """Model-based: a random interleaving of single pushes (in any order, running ahead into the
    next iteration for units that have already launched), pulls (some of them before the key's
    unit can launch) and learning-rate changes between iterations, mirrored on the oracle."""
    import torch
    r = _rng(4242, seed)
    numel = [int(x) for x in r.choice([1, 7, 64, 300, 1024, 1500, 4096, 5000, 9000], size=int(r.integers(3, 12)))]
    K, W = len(numel), int(r.choice([1, 2, 3, 8]))
    dtype = "f32" if seed % 2 == 0 else "f16"
    bucket = int(r.choice([1, 4096, 16384, 1 << 30]))
    pair = Pair(numel, W, dtype, bucket, lr=0.1, momentum=0.9, wd=1e-4, descending=bool(seed % 3 == 0))
    try:
        pair.set_weights([_rng(seed, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
        plan = pair.gpu.plan
        unit_of = [plan.key(k)[0] for k in range(K)]
        pulls = []                                   # (tensor, expected values)
        keep = []
        iters = 4
        pushed_in_iter = [0] * K                     # how many iterations each key has been pushed for
        launched_iter = [0] * plan.num_units         # how many times each unit has launched (model of the chain)
        pending = [set() for _ in range(plan.num_units)]
        U = plan.num_units
        order_units = list(range(U - 1, -1, -1)) if seed % 3 == 0 else list(range(U))
        pos = 0                                      # position of the chain in order_units
        steps = 0
        while min(pushed_in_iter) < iters and steps < 10000:
            steps += 1
            k = int(r.integers(0, K))
            u = unit_of[k]
            can_push = pushed_in_iter[k] < iters and k not in pending[u] and pushed_in_iter[k] == launched_iter[u]
            if can_push:
                t = pushed_in_iter[k]
                g = [(_rng(seed, 7, t, k, rr).standard_normal(numel[k], dtype=F) * F(0.01)) for rr in range(W)]
                if dtype == "f16":
                    g = [x.astype(np.float16) for x in g]
                dev = [to_device(x) for x in g]
                keep.append(dev)
                pair.gpu.push(k, dev)
                pair.cpu.step_one_key(k, g)
                pushed_in_iter[k] += 1
                pending[u].add(k)
                keys_of_u = set(plan.unit(u)[0])
                # model of the chain: launch while the unit at the chain position is complete
                while pending[order_units[pos]] == set(plan.unit(order_units[pos])[0]):
                    uu = order_units[pos]
                    pending[uu] = set()
                    launched_iter[uu] += 1
                    pos = (pos + 1) % U
            if r.random() < 0.3:
                kk = int(r.integers(0, K))
                out = torch.zeros(numel[kk], device="cuda")
                pair.gpu.pull(kk, out)               # may be queued behind the key's launch
                pulls.append((out, pair.cpu.w[kk].copy()))
        assert min(pushed_in_iter) == iters, "the model got stuck"
        pair.gpu.wait()
        total, log = pair.gpu.launch_log()
        assert sum(n for _, n in log) == U * iters
        for out, ref in pulls:
            assert np.array_equal(out.cpu().numpy().view(np.uint32), ref.view(np.uint32))
        pair.compare(f"random session {seed}")
    finally:
        pair.close()


def test_maximum_rank_count_and_many_keys():
    """W = 256 (the library's maximum) through the run-time-W kernel, and a store of 3000 small keys."""
    numel = [5, 1030, 64]
    for order in (orc.SEQUENTIAL, orc.PAIRWISE):
        pair = Pair(numel, 256, "f16", 4096, lr=0.1, momentum=0.9, wd=1e-4, order=order)
        try:
            pair.set_weights([_rng(11, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)])
            pair.step(_grads(numel, 256, "f16", 1100))
            pair.compare(f"W=256 order {order}")
        finally:
            pair.close()
    r = _rng(12)
    numel = [int(x) for x in r.integers(0, 300, size=3000)]
    pair = Pair(numel, 2, "f32", 8192, lr=0.1, momentum=0.9, wd=1e-4, keep_sum=False)
    try:
        assert pair.gpu.plan.num_units > 50
        g = [[(_rng(13, k, rr).standard_normal(n, dtype=F) * F(0.01)) for rr in range(2)] for k, n in enumerate(numel)]
        import torch
        flat = [torch.from_numpy(np.concatenate([gk[rr] for gk in g])).cuda() for rr in range(2)]
        offs = np.concatenate([[0], np.cumsum(numel)])
        dev = [[flat[rr][offs[k]:offs[k + 1]] for rr in range(2)] for k in range(len(numel))]   # views, mostly misaligned
        pair.step(g, dev=dev)
        pair.step(g, dev=dev, mode="each", order=[int(x) for x in r.permutation(len(numel))])
        import torch
        outs = [torch.empty(n, device="cuda") for n in numel]
        pair.gpu.pull_list(list(range(len(numel))), outs)
        pair.gpu.wait()
        for k in range(len(numel)):
            assert np.array_equal(outs[k].cpu().numpy().view(np.uint32), pair.cpu.w[k].view(np.uint32)), k
    finally:
        pair.close()


def test_init_rejects_bad_arguments():
    kv = pytest.importorskip("paper_1802_06949_amd")
    for kwargs in (dict(W=0), dict(W=257), dict(reduce_order=2), dict(unroll=3), dict(nontemporal=2), dict(lane_elems=3),
                   dict(lane_elems=2, unroll=4), dict(resident_workgroups=2), dict(resident_workgroups=9),
                   dict(autotune=True, unroll=2)):
        args = dict(W=2, lr=0.1)
        args.update(kwargs)
        with pytest.raises(kv.KVError) as e:
            kv.KVStore([10, 20], args.pop("W"), "f32", 4096, **args)
        assert e.value.status == -1, kwargs
    with pytest.raises(kv.KVError):
        kv.KVStore([], 2, "f32", 4096, lr=0.1)
    with pytest.raises(kv.KVError):
        kv.KVStore([10, -5], 2, "f32", 4096, lr=0.1)
    with pytest.raises(kv.KVError):
        kv.KVStore([10], 2, "f32", 0, lr=0.1)


def test_tuning_values_round_trip_and_bad_ones_are_refused():
    import paper_1802_06949_amd as kv
    want = dict(unroll=2, workgroups_per_cu=3, nontemporal=5, xcd_remap=128, lane_elems=2, resident_workgroups=6, run_time_w=1)
    st = kv.KVStore([1000, 5000], 4, "f32", 1 << 12, lr=0.1, **want)
    try:
        got, settled = st.get_tuning()
        assert got == want and settled
    finally:
        st.close()
    st = kv.KVStore([1000, 5000], 4, "f32", 1 << 12, lr=0.1)            # defaults resolved, never the "default" codes
    try:
        got, _ = st.get_tuning()
        assert got["unroll"] == 1 and got["lane_elems"] in (1, 2, 4) and got["nontemporal"] in (9, 13)
        assert got["workgroups_per_cu"] == 0 and got["xcd_remap"] in (64, 1024) and got["resident_workgroups"] in (0, 3, 4, 5, 6, 7, 8)
    finally:
        st.close()
    for bad in (dict(workgroups_per_cu=65), dict(xcd_remap=(1 << 20) + 1), dict(resident_workgroups=2), dict(resident_workgroups=9),
                dict(resident_workgroups=-1), dict(nontemporal=2), dict(lane_elems=3), dict(lane_elems=2, unroll=4), dict(run_time_w=2),
                dict(run_time_w=-1)):
        with pytest.raises(kv.KVError) as e:
            kv.KVStore([1000], 4, "f32", 1 << 12, lr=0.1, **bad)
        assert e.value.status == -1, bad
