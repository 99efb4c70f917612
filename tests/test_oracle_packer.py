"""Pins of the oracle's bucket-packing scan and of the key-set generators.

Expected plans are worked out by hand from the policy: a key of size
numel * itemsize (one gradient copy) is small iff size < bucket_bytes; small keys
join the open bucket while it stays <= bucket_bytes; a large key is a unit of its
own and leaves the open bucket open; units are numbered by their first key.
"""
from __future__ import annotations

import pytest

import workloads as wl
from oracle import kv_oracle as orc


def _plan(numel, itemsize, bucket):
    return [(u.keys, u.large) for u in orc.plan_units(numel, itemsize, bucket)]


def test_large_keys_do_not_close_the_open_bucket():
    # sizes in bytes: 40, 1200 (large), 20, 1024 (== bucket: large), 80, 4
    numel = [10, 300, 5, 256, 20, 1]
    assert _plan(numel, 4, 1024) == [([0, 2, 4, 5], False), ([1], True), ([3], True)]
    units = orc.plan_units(numel, 4, 1024)
    # key starts are multiples of 64 elements (256 bytes):
    # unit 0: k0 @0..10, k2 @64..69, k4 @128..148, k5 @192..193; unit 1: k1 @256..556; unit 2: k3 @576
    assert orc.arena_offsets(numel, units) == [0, 256, 64, 576, 128, 192]
    # with 16-byte alignment: k2 @12..17, k4 @20..40, k5 @40..41; k1 @44..344; k3 @344
    assert orc.arena_offsets(numel, units, align_elems=4) == [0, 44, 12, 344, 20, 40]


def test_bucket_closes_on_overflow_and_accepts_exact_fit():
    assert _plan([100, 100, 100, 50, 7], 4, 1000) == [([0, 1], False), ([2, 3, 4], False)]
    assert _plan([125, 125, 1], 4, 1000) == [([0, 1], False), ([2], False)]


def test_extreme_bucket_sizes():
    numel = [3, 1, 4, 1, 5, 9, 2, 6]
    assert _plan(numel, 4, 1) == [([k], True) for k in range(len(numel))]
    assert _plan(numel, 4, 1 << 40) == [(list(range(len(numel))), False)]


def test_itemsize_counts_one_gradient_copy():
    # 300 halves = 600 B < 1024 (small); 300 floats = 1200 B (large)
    assert _plan([300, 10], 2, 1024) == [([0, 1], False)]
    assert _plan([300, 10], 4, 1024) == [([0], True), ([1], False)]


# Published parameter counts of the public architectures (ResNet-50: 25 557 032,
# VGG-16: 138 357 544) and the unit counts that follow from the policy.
@pytest.mark.parametrize("cfg_id,keys,params,small,large", [
    (1, 4, 203_530, 1, 1),
    (2, 65, 272_474, 6, 0),
    (3, 161, 25_557_032, 12, 10),
    (4, 161, 25_557_032, 8, 0),
    (5, 32, 138_357_544, 7, 2),
    (6, 209, 11_194_984, 12, 0),          # Inception-BN-shaped; count follows from the layer table, not pinned
])
def test_benchmark_key_sets(cfg_id, keys, params, small, large):
    cfg = wl.get_config(cfg_id)
    assert len(cfg.keys) == keys and cfg.total_numel == params
    units = orc.plan_units(cfg.numel, cfg.grad_itemsize, cfg.bucket_bytes)
    assert sum(not u.large for u in units) == small
    assert sum(u.large for u in units) == large
    assert sorted(k for u in units for k in u.keys) == list(range(keys))
    assert [u.keys[0] for u in units] == sorted(u.keys[0] for u in units)


def test_resnet50_has_keys_of_exactly_one_bucket():
    cfg = wl.get_config(3)
    exact = [k for k, n in enumerate(cfg.numel) if n * 4 == cfg.bucket_bytes]
    assert len(exact) == 5
    units = orc.plan_units(cfg.numel, 4, cfg.bucket_bytes)
    for k in exact:
        assert any(u.large and u.keys == [k] for u in units)


def test_generators_are_seeded_and_independent_per_rank():
    import numpy as np
    cfg = wl.get_config(2)
    a = wl.make_gradient(cfg, 0, 3, 1)
    assert np.array_equal(a, wl.make_gradient(cfg, 0, 3, 1))
    assert not np.array_equal(a, wl.make_gradient(cfg, 0, 3, 2))
    assert not np.array_equal(a, wl.make_gradient(cfg, 1, 3, 1))
    cfg3 = wl.get_config(3)
    z = wl.zero_keys(cfg3)
    assert len(z) == 8
    k = sorted(z)[0]
    assert not wl.make_gradient(cfg3, 0, k, 5).any()
    s = wl.key_sigma(cfg3)
    assert s.min() >= 1e-4 * 0.999 and s.max() <= 1e-2 * 1.001
    assert wl.make_gradient(wl.get_config(4), 0, 0, 0).dtype == np.float16


def test_learning_rate_scaling_goes_through_the_papers_two_points():
    # Evaluation section: 0.1 by default, 1.0 at 256 GPUs, grown linearly with the mini-batch
    assert wl.scaled_lr(1) == 0.1 and wl.scaled_lr(8) == 0.1
    assert wl.scaled_lr(256) == 1.0 and wl.scaled_lr(128) == 0.5
