"""Pins of the CPU oracle against what the paper and the arithmetic fix.

None of these tests touches the GPU library.  They are chosen so that a
plausible mistake in the oracle (a dropped term, a wrong sign, w and m swapped,
a wrong fold order or tree shape, an inexact half conversion, a fused
multiply-add) fails at least one of them.
"""
from __future__ import annotations

import math

import numpy as np
import pytest

from oracle import kv_oracle as orc
from tests.helpers import bits_equal, load_hand_cases, numpy_step, within_tol

F = np.float32


def _rng(*seed):
    return np.random.Generator(np.random.SFC64(list(seed)))


# ---------------------------------------------------------------- paper snippet
@pytest.mark.parametrize("W", [1, 2, 3, 4, 5, 7, 8, 9, 16, 32])
@pytest.mark.parametrize("order", [orc.SEQUENTIAL, orc.PAIRWISE])
def test_kvstore_snippet_ones(W, order):
    """KVStore API section: every worker pushes ones((2,3)); the pulled value is
    the aggregate over all workers, W * ones((2,3))."""
    g = [np.ones(6, dtype=F) for _ in range(W)]
    s = orc.reduce_key(g, order)
    assert bits_equal(s, np.full(6, W, dtype=F))


# ---------------------------------------------------------------- hand cases
@pytest.mark.parametrize("case", load_hand_cases(), ids=lambda c: c["name"])
def test_hand_computed_cases(case):
    dt = np.float32 if case["dtype"] == "f32" else np.float16
    g = [np.array(r, dtype=dt) for r in case["g"]]
    W = len(g)
    st = orc.OracleStore([len(case["w"])], W, lr=case["lr"], momentum=case["momentum"], wd=case["wd"],
                         rescale=case["rescale"], order=case["order"], keep_sum=True)
    st.set_weights(0, np.array(case["w"], dtype=F))
    st.set_momentum(0, np.array(case["m"], dtype=F))
    st.step([g])
    assert np.array_equal(st.s[0], np.array(case["expect_s"], dtype=F))
    assert np.array_equal(st.m[0], np.array(case["expect_m"], dtype=F))
    assert np.array_equal(st.w[0], np.array(case["expect_w"], dtype=F))
    # the raw-sum entry point agrees with the fused one
    assert bits_equal(orc.reduce_key(g, case["order"]), st.s[0])


# ---------------------------------------------------------------- half widening
def test_half_widening_matches_numpy_on_all_bit_patterns():
    """With W = 1 the sum is g_0 itself, so the output is the widened input.
    numpy's float16 -> float32 cast is the library routine it must equal,
    bit for bit, on all 65 536 patterns (zeros, subnormals, inf, nan payloads)."""
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16).view(np.float16)
    s = orc.reduce_key([h], orc.SEQUENTIAL)
    with np.errstate(invalid="ignore"):
        ref = h.astype(np.float32)
    assert np.array_equal(s.view(np.uint32), ref.view(np.uint32))


def test_rounding_to_half_matches_numpy():
    """The fp16 replicas of the weights are binary32 values rounded to nearest-even binary16.
    numpy's float32 -> float16 cast is the library routine: every half round-trips, and every
    midpoint between neighbouring halves (the ties), its two binary32 neighbours, the overflow
    threshold, the subnormal range and three million random values agree bit for bit."""
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = h.view(np.float16).astype(np.float32)
    ok = ~np.isnan(f)
    assert np.array_equal(orc.round_to_half(f).view(np.uint16)[ok], h[ok])
    assert np.all(np.isnan(orc.round_to_half(f[~ok])))
    fin = np.unique(f[np.isfinite(f)])
    mid = ((fin[:-1].astype(np.float64) + fin[1:].astype(np.float64)) / 2).astype(F)      # exact in binary32
    special = np.array([65519.996, 65520, 65504, 65535, 1e9, -1e9, 2.0 ** -25, np.nextafter(F(2.0 ** -25), F(1)),
                        1.5 * 2.0 ** -24, 2.0 ** -14, np.nextafter(F(2.0 ** -14), F(0)), 0.0, -0.0, np.inf, -np.inf], dtype=F)
    cands = np.concatenate([mid, np.nextafter(mid, F(np.inf)), np.nextafter(mid, F(-np.inf)), special, -mid])
    with np.errstate(over="ignore"):
        assert np.array_equal(orc.round_to_half(cands).view(np.uint16), cands.astype(np.float16).view(np.uint16))
    r = _rng(99)
    x = r.standard_normal(3_000_000, dtype=F) * (F(10.0) ** r.integers(-9, 6, 3_000_000).astype(F))
    with np.errstate(over="ignore"):
        assert np.array_equal(orc.round_to_half(x).view(np.uint16), x.astype(np.float16).view(np.uint16))


# ---------------------------------------------------------------- identical copies
@pytest.mark.parametrize("W", [2, 4, 8, 16, 32])
def test_identical_copies_pairwise_power_of_two_exact(W):
    g = (_rng(1, W).standard_normal(200_000, dtype=F) * F(0.01)).astype(F)
    s = orc.reduce_key([g] * W, orc.PAIRWISE)
    assert bits_equal(s, F(W) * g)          # scaling by a power of two is exact


@pytest.mark.parametrize("W", [2, 4])
def test_identical_copies_left_fold_small_W_exact(W):
    g = (_rng(2, W).standard_normal(200_000, dtype=F) * F(0.01)).astype(F)
    s = orc.reduce_key([g] * W, orc.SEQUENTIAL)
    assert bits_equal(s, F(W) * g)


@pytest.mark.parametrize("W", [8, 16, 32])
def test_identical_copies_left_fold_exact_when_low_bits_clear(W):
    """k*g is representable for every k <= W once the low log2(W) mantissa bits of
    g are zero, so the left fold is exact too."""
    g = (_rng(3, W).standard_normal(200_000, dtype=F) * F(0.01)).astype(F)
    mask = np.uint32(0xFFFFFFFF) << np.uint32(int(math.log2(W)))
    g = (g.view(np.uint32) & mask).view(F)
    s = orc.reduce_key([g] * W, orc.SEQUENTIAL)
    assert bits_equal(s, F(W) * g)


def test_left_fold_of_eight_copies_is_a_left_fold():
    """For generic fp32 data a left fold of 8 identical copies is NOT 8*g on a
    large share of elements (3g, 5g, 6g, 7g need extra mantissa bits), while a
    tree is always exact.  An oracle that secretly used a tree, or accumulated in
    double, would return 8*g everywhere."""
    g = (_rng(4).standard_normal(400_000, dtype=F) * F(0.01)).astype(F)
    s = orc.reduce_key([g] * 8, orc.SEQUENTIAL)
    frac = float(np.mean(s != F(8) * g))
    assert 0.25 < frac < 0.65
    rel = np.abs(s.astype(np.float64) - 8.0 * g.astype(np.float64)) / np.abs(8.0 * g.astype(np.float64))
    assert float(rel.max()) <= 7 * 2.0 ** -24


@pytest.mark.parametrize("W", [2, 3, 5, 7, 8, 16, 32])
@pytest.mark.parametrize("order", [orc.SEQUENTIAL, orc.PAIRWISE])
def test_identical_half_copies_always_exact(W, order):
    g = (_rng(5, W).standard_normal(100_000, dtype=F) * F(0.01)).astype(np.float16)
    s = orc.reduce_key([g] * W, order)
    assert np.array_equal(s.astype(np.float64), W * g.astype(np.float64))


# ---------------------------------------------------------------- error bound vs exact sum
@pytest.mark.parametrize("W", [2, 3, 8, 13, 32])
@pytest.mark.parametrize("order", [orc.SEQUENTIAL, orc.PAIRWISE])
def test_sum_within_bound_of_exact_sum(W, order):
    n = 20_000
    g = [(_rng(6, W, r).standard_normal(n, dtype=F) * F(0.01)).astype(F) for r in range(W)]
    s = orc.reduce_key(g, order).astype(np.float64)
    g64 = np.stack([x.astype(np.float64) for x in g])          # binary64 holds these sums to ~1e-16
    exact = np.array([math.fsum(g64[:, i]) for i in range(n)])
    depth = W - 1 if order == orc.SEQUENTIAL else math.ceil(math.log2(W))
    bound = depth * 2.0 ** -24 * np.abs(g64).sum(axis=0) * 1.0001
    assert np.all(np.abs(s - exact) <= bound)


def test_half_sums_exact_and_order_free():
    """Halves are multiples of 2^-24; while every partial sum stays below 1 it is
    representable in binary32, so any order gives the exact sum."""
    W, n = 32, 50_000
    g = [(_rng(7, r).standard_normal(n, dtype=F) * F(0.005)).astype(np.float16) for r in range(W)]
    g64 = np.stack([x.astype(np.float64) for x in g])
    assert float(np.abs(g64).sum(axis=0).max()) < 1.0
    exact = g64.sum(axis=0)
    for order in (orc.SEQUENTIAL, orc.PAIRWISE):
        assert np.array_equal(orc.reduce_key(g, order).astype(np.float64), exact)
    perm = _rng(8).permutation(W)
    assert bits_equal(orc.reduce_key([g[p] for p in perm]), orc.reduce_key(g))


# ---------------------------------------------------------------- update closed forms
def _store(n, W, **kw):
    return orc.OracleStore([n], W, **kw)


def test_plain_sgd_is_w_minus_lr_mean_gradient():
    """eq. (1) with the averaged gradient: momentum = wd = 0 => w' = w - lr*mean(g)."""
    W, n, lr = 8, 50_000, 0.1
    g = [(_rng(9, r).standard_normal(n, dtype=F) * F(0.01)).astype(F) for r in range(W)]
    w0 = _rng(10).standard_normal(n, dtype=F)
    st = _store(n, W, lr=lr, momentum=0.0, wd=0.0)
    st.set_weights(0, w0)
    st.set_momentum(0, _rng(11).standard_normal(n, dtype=F))     # must be ignored when momentum = 0
    st.step([g])
    mean64 = np.stack([x.astype(np.float64) for x in g]).mean(axis=0)
    ref = w0.astype(np.float64) - float(F(lr)) * mean64
    assert within_tol(st.w[0], ref, 1e-6)
    # dw itself is a cancelling sum: bound its error by the left fold's (W-1) roundings on sum|g|
    # plus the roundings of the scale and the lr product
    dw64 = -float(F(lr)) * mean64
    abs_sum = np.abs(np.stack([x.astype(np.float64) for x in g])).sum(axis=0)
    bound = float(F(lr)) / W * (W - 1) * 2.0 ** -24 * abs_sum + 3 * 2.0 ** -24 * np.abs(dw64)
    assert np.all(np.abs(st.m[0].astype(np.float64) - dw64) <= bound)


def test_zero_lr_from_rest_leaves_weights_untouched():
    W, n = 4, 10_000
    g = [_rng(12, r).standard_normal(n, dtype=F) for r in range(W)]
    w0 = _rng(13).standard_normal(n, dtype=F)
    st = _store(n, W, lr=0.0, momentum=0.9, wd=1e-4)
    st.set_weights(0, w0)
    st.step([g])
    assert bits_equal(st.w[0], w0)
    assert np.all(st.m[0] == 0)


def test_zero_lr_with_momentum_state():
    W, n, mu = 4, 10_000, 0.9
    g = [_rng(14, r).standard_normal(n, dtype=F) for r in range(W)]
    w0 = _rng(15).standard_normal(n, dtype=F)
    m0 = _rng(16).standard_normal(n, dtype=F)
    st = _store(n, W, lr=0.0, momentum=mu, wd=1e-4)
    st.set_weights(0, w0); st.set_momentum(0, m0)
    st.step([g])
    assert bits_equal(st.m[0], F(mu) * m0)
    assert bits_equal(st.w[0], w0 + F(mu) * m0)


def test_zero_gradients_still_decay_and_coast():
    """g = 0 on every rank: w' = w + mu*m - lr*wd*w (weight decay and momentum act)."""
    W, n, lr, mu, wd = 8, 10_000, 0.1, 0.9, 1e-2
    g = [np.zeros(n, dtype=F) for _ in range(W)]
    w0 = _rng(17).standard_normal(n, dtype=F)
    m0 = _rng(18).standard_normal(n, dtype=F) * F(0.01)
    st = _store(n, W, lr=lr, momentum=mu, wd=wd)
    st.set_weights(0, w0); st.set_momentum(0, m0)
    st.step([g])
    w64, m64 = w0.astype(np.float64), m0.astype(np.float64)
    dw = float(F(mu)) * m64 - float(F(lr)) * float(F(wd)) * w64
    # two cancelling terms: bound the error by a few roundings on their magnitudes
    u = 2.0 ** -24
    bound_m = 3 * u * (np.abs(float(F(mu)) * m64) + np.abs(float(F(lr)) * float(F(wd)) * w64))
    assert np.all(np.abs(st.m[0].astype(np.float64) - dw) <= bound_m)
    assert np.all(np.abs(st.w[0].astype(np.float64) - (w64 + dw)) <= bound_m + u * np.abs(w64 + dw))
    assert not bits_equal(st.w[0], w0)


def test_single_worker_matches_library_momentum_sgd_trajectory():
    """W = 1, rescale = 1 is a textbook single-worker momentum-SGD step.  With a
    constant learning rate torch.optim.SGD (buf = mu*buf + g + wd*w; w -= lr*buf)
    follows the same trajectory with m = -lr*buf; it runs in float64 here."""
    torch = pytest.importorskip("torch")
    n, lr, mu, wd, steps = 5_000, 0.125, 0.875, 2.0 ** -7, 6     # exactly representable
    w0 = _rng(19).standard_normal(n, dtype=F)
    st = _store(n, 1, lr=lr, momentum=mu, wd=wd, rescale=1.0)
    st.set_weights(0, w0)
    p = torch.nn.Parameter(torch.from_numpy(w0.astype(np.float64)))
    opt = torch.optim.SGD([p], lr=lr, momentum=mu, weight_decay=wd, dampening=0.0, nesterov=False)
    for t in range(steps):
        g = _rng(20, t).standard_normal(n, dtype=F) * F(0.05)
        st.step([[g]])
        p.grad = torch.from_numpy(g.astype(np.float64))
        opt.step()
    buf = opt.state[p]["momentum_buffer"].numpy()
    # binary32 roundings accumulate over the steps; a different update form is off by >= 1e-2
    assert np.allclose(st.w[0], p.detach().numpy(), rtol=1e-5, atol=1e-7)
    assert np.allclose(st.m[0], -lr * buf, rtol=1e-4, atol=1e-7)


def test_default_rescale_is_one_over_W():
    W, n = 8, 1000
    g = [_rng(21, r).standard_normal(n, dtype=F) for r in range(W)]
    a = _store(n, W, lr=0.1, momentum=0.9, wd=0.0)
    b = _store(n, W, lr=0.1, momentum=0.9, wd=0.0, rescale=0.125)
    a.step([g]); b.step([g])
    assert bits_equal(a.w[0], b.w[0]) and bits_equal(a.m[0], b.m[0])


# ---------------------------------------------------------------- IEEE corner cases
def test_negative_zero_sum_keeps_its_sign():
    g = [np.full(4, -0.0, dtype=F) for _ in range(5)]
    for order in (orc.SEQUENTIAL, orc.PAIRWISE):
        s = orc.reduce_key(g, order)
        assert np.all(s.view(np.uint32) == 0x80000000)


def test_subnormals_are_kept():
    tiny = np.array([1], dtype=np.uint32).view(F)            # 2^-149
    s = orc.reduce_key([np.repeat(tiny, 3)] * 4)
    assert np.all(s.view(np.uint32) == 4)
    st = _store(3, 4, lr=1.0, momentum=0.0, wd=0.0, rescale=1.0)
    st.step([[np.repeat(tiny, 3)] * 4])
    assert np.all(st.m[0].view(np.uint32) == (0x80000000 | 4))


def test_nan_and_inf_propagate():
    g0 = np.array([np.inf, np.nan, 1.0, np.inf], dtype=F)
    g1 = np.array([1.0, 1.0, 1.0, -np.inf], dtype=F)
    s = orc.reduce_key([g0, g1])
    assert s[0] == np.inf and np.isnan(s[1]) and s[2] == 2.0 and np.isnan(s[3])


def test_each_operation_rounds_once():
    """momentum*m - lr*t with the product fused into the subtraction keeps bits that
    two roundings drop.  With a = 1 + 2^-12: mu*m = a*a = 1 + 2^-11 + 2^-24, a tie
    that rounds to 1 + 2^-11; lr*t = 1 + 2^-11; so dw = 0 with one rounding per
    operation, and 2^-24 with a fused multiply-add."""
    a = F(1 + 2.0 ** -12)
    w0 = np.array([a], dtype=F)
    st = _store(1, 1, lr=1.0, momentum=float(a), wd=0.0, rescale=1.0)
    st.set_weights(0, np.array([0.0], dtype=F))
    st.set_momentum(0, w0)                       # mu*m = a*a = 1 + 2^-11 + 2^-24 -> 1 + 2^-11
    g = np.array([1 + 2.0 ** -11], dtype=F)      # lr*t = 1 + 2^-11
    st.step([[g]])
    assert st.m[0][0] == 0.0                     # fused: 2^-24 would survive
    s, wn, mn = numpy_step([g], np.array([0.0], dtype=F), w0, rescale=1.0, lr=1.0, momentum=float(a), wd=0.0)
    assert bits_equal(st.m[0], mn)


# ---------------------------------------------------------------- invariants
@pytest.mark.parametrize("W", [1, 2, 3])
def test_orders_coincide_up_to_three_ranks(W):
    g = [_rng(22, W, r).standard_normal(10_000, dtype=F) for r in range(W)]
    assert bits_equal(orc.reduce_key(g, orc.SEQUENTIAL), orc.reduce_key(g, orc.PAIRWISE))


def test_orders_differ_on_generic_data_at_eight_ranks():
    g = [_rng(23, r).standard_normal(50_000, dtype=F) for r in range(8)]
    assert not bits_equal(orc.reduce_key(g, orc.SEQUENTIAL), orc.reduce_key(g, orc.PAIRWISE))


def test_rank_permutation_moves_left_fold_only_within_bound():
    W, n = 8, 50_000
    g = [_rng(24, r).standard_normal(n, dtype=F) for r in range(W)]
    a = orc.reduce_key(g).astype(np.float64)
    b = orc.reduce_key(g[::-1]).astype(np.float64)
    assert np.any(a != b)
    bound = 2 * (W - 1) * 2.0 ** -24 * np.abs(np.stack(g).astype(np.float64)).sum(axis=0)
    assert np.all(np.abs(a - b) <= bound)


def test_threaded_ranges_are_bit_identical_and_deterministic():
    W, n = 4, 300_000
    g = [_rng(25, r).standard_normal(n, dtype=F) * F(0.01) for r in range(W)]
    w0 = _rng(26).standard_normal(n, dtype=F)
    outs = []
    for threads in (1, 4, 1):
        st = _store(n, W, lr=0.1, momentum=0.9, wd=1e-4)
        st.set_weights(0, w0)
        for _ in range(3):
            st.step([g], threads=threads)
        outs.append((st.w[0].copy(), st.m[0].copy()))
    for w, m in outs[1:]:
        assert bits_equal(w, outs[0][0]) and bits_equal(m, outs[0][1])


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("order", [orc.SEQUENTIAL, orc.PAIRWISE])
def test_numpy_float32_cross_check_three_steps(dtype, order):
    """Third evaluation of the same step (vectorised numpy float32), bitwise."""
    W, numel = 5, [1, 7, 64, 1000, 4099]
    lr, mu, wd = 0.1, 0.9, 1e-4
    st = orc.OracleStore(numel, W, lr=lr, momentum=mu, wd=wd, order=order, keep_sum=True)
    w = [_rng(27, k).standard_normal(n, dtype=F) for k, n in enumerate(numel)]
    m = [np.zeros(n, dtype=F) for n in numel]
    for k in range(len(numel)):
        st.set_weights(k, w[k])
    for t in range(3):
        grads = []
        for k, n in enumerate(numel):
            gk = [_rng(28, t, k, r).standard_normal(n, dtype=F) * F(0.01) for r in range(W)]
            if dtype == "f16":
                gk = [x.astype(np.float16) for x in gk]
            grads.append(gk)
        st.step(grads)
        for k in range(len(numel)):
            s, w[k], m[k] = numpy_step(grads[k], w[k], m[k], rescale=float(F(1) / F(W)), lr=lr, momentum=mu,
                                       wd=wd, order=order)
            assert bits_equal(st.s[k], s)
            assert bits_equal(st.w[k], w[k]) and bits_equal(st.m[k], m[k])
