"""CPU-only tests of the built library: exported symbols, the bucket plan against
the oracle's plain scan, and the launch-order chain.  No compute call is made."""
from __future__ import annotations

import ctypes
import os
import re

import numpy as np
import pytest

import workloads as wl
from oracle import kv_oracle as orc

kv = pytest.importorskip("paper_1802_06949_amd")
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _rng(*seed):
    return np.random.Generator(np.random.SFC64(list(seed)))


def _declared(*headers):
    names = set()
    for h in headers:
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(kv_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    names = _declared("kv.h", "kv_engine.h", "kv_diag.h")
    assert len(names) >= 30
    lib = ctypes.CDLL(kv.library_path())
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/kv.h but not exported"


def test_binding_covers_every_declared_symbol():
    src = open(os.path.join(ROOT, "paper_1802_06949_amd", "kvstore.py")).read()
    src += open(os.path.join(ROOT, "paper_1802_06949_amd", "engine.py")).read()
    for n in _declared("kv.h", "kv_engine.h", "kv_diag.h"):
        assert f'"{n}"' in src or f"L.{n}" in src, f"{n} has no ctypes signature in the binding"


def _lib_plan(numel, dtype, bucket):
    p = kv.Plan(numel, dtype, bucket)
    return p, p.units()


@pytest.mark.parametrize("cfg_id", [1, 2, 3, 4, 5, 6])
def test_plan_matches_oracle_scan_on_benchmark_configs(cfg_id):
    cfg = wl.get_config(cfg_id)
    p, units = _lib_plan(cfg.numel, cfg.grad_dtype, cfg.bucket_bytes)
    ref = orc.plan_units(cfg.numel, cfg.grad_itemsize, cfg.bucket_bytes)
    assert units == [(u.keys, u.large) for u in ref]
    off = orc.arena_offsets(cfg.numel, ref)
    assert [p.key(k)[1] for k in range(len(cfg.numel))] == off
    assert [p.key(k)[0] for k in range(len(cfg.numel))] == [i for k in range(len(cfg.numel))
                                                            for i, u in enumerate(ref) if k in u.keys]
    assert p.arena_numel >= max(o + n for o, n in zip(off, cfg.numel))


@pytest.mark.parametrize("seed", range(40))
def test_plan_matches_oracle_scan_on_random_key_sets(seed):
    r = _rng(77, seed)
    K = int(r.integers(1, 60))
    numel = [int(x) for x in r.choice([0, 1, 3, 10, 64, 100, 255, 256, 257, 1000, 4096, 5000, 70000], size=K)]
    dtype = ["f32", "f16"][seed % 2]
    bucket = int(r.choice([1, 2, 4, 40, 1024, 1028, 4096, 16384, 1 << 20, 1 << 40]))
    p, units = _lib_plan(numel, dtype, bucket)
    ref = orc.plan_units(numel, 4 if dtype == "f32" else 2, bucket)
    assert units == [(u.keys, u.large) for u in ref]
    assert [p.key(k)[1] for k in range(K)] == orc.arena_offsets(numel, ref)


@pytest.mark.parametrize("seed", range(10))
def test_keys_start_on_256_byte_boundaries_and_never_overlap(seed):
    """Stated on its own, not through the oracle's mirror of the layout: every key of the arena starts on a multiple
    of 64 fp32 elements, keys lie in unit order without overlapping, and the arena ends on such a boundary."""
    r = _rng(78, seed)
    K = int(r.integers(1, 80))
    numel = [int(x) for x in r.choice([0, 1, 3, 10, 63, 64, 65, 100, 1000, 4097, 70001], size=K)]
    p, units = _lib_plan(numel, "f32", int(r.choice([1, 1024, 1 << 20])))
    order = [k for keys, _ in units for k in keys]
    end = 0
    for k in order:
        off = p.key(k)[1]
        assert off % 64 == 0 and off >= end, (k, off, end)
        end = off + numel[k]
    assert p.arena_numel >= end and p.arena_numel % 64 == 0


def test_plan_rejects_bad_arguments():
    for args in [([], "f32", 1024), ([10, -1], "f32", 1024), ([10], "f32", 0)]:
        with pytest.raises(kv.KVError) as e:
            kv.Plan(*args)
        assert e.value.status == -1
    with pytest.raises(ValueError):
        kv.Plan([10], "f64", 1024)


@pytest.mark.parametrize("seed", range(20))
def test_chain_runs_ascend_whatever_the_push_order(seed):
    """The paper's ordering requirement: the order in which units run is the same
    whatever order the gradients become ready in."""
    r = _rng(78, seed)
    cfg = wl.get_config(int(r.integers(1, 7)))
    p = kv.Plan(cfg.numel, cfg.grad_dtype, cfg.bucket_bytes)
    c = kv.Chain(p)
    K, U = p.num_keys, p.num_units
    for it in range(3):
        covered = []
        for k in r.permutation(K):
            assert c.mark(int(k)) == 0
            for first, n in c.drain():
                assert n >= 1
                covered += list(range(first, first + n))
                # a unit only runs once all its keys are in
            assert covered == list(range(len(covered)))
        assert covered == list(range(U))
        assert c.pending_keys == 0 and c.next_unit == 0


@pytest.mark.parametrize("seed", range(10))
def test_descending_chain_runs_from_the_last_unit_down(seed):
    r = _rng(79, seed)
    cfg = wl.get_config(int(r.integers(1, 7)))
    p = kv.Plan(cfg.numel, cfg.grad_dtype, cfg.bucket_bytes)
    c = kv.Chain(p)
    assert c.set_descending(True) == 0
    K, U = p.num_keys, p.num_units
    for it in range(2):
        covered = []
        for k in r.permutation(K):
            assert c.mark(int(k)) == 0
            for lowest, n in c.drain():
                covered += list(range(lowest + n - 1, lowest - 1, -1))
        assert covered == list(range(U - 1, -1, -1))
    # keys pushed last layer first (the order a backward pass produces them): every unit
    # launches as soon as its own keys are in
    launches = []
    for k in range(K - 1, -1, -1):
        c.mark(k)
        launches += c.drain()
    assert len(launches) == U and all(n == 1 for _, n in launches)
    assert c.mark(0) == 0 and c.set_descending(False) == -3          # not in the middle of an iteration


def test_chain_in_order_list_is_one_run():
    cfg = wl.get_config(3)
    p = kv.Plan(cfg.numel, cfg.grad_dtype, cfg.bucket_bytes)
    c = kv.Chain(p)
    for k in range(p.num_keys):
        assert c.mark(k) == 0
    assert c.drain() == [(0, p.num_units)]


def test_chain_rejects_second_push_until_the_unit_ran():
    p = kv.Plan([16, 4096, 16], "f32", 1024)            # unit 0 = {0, 2}, unit 1 = {1}
    c = kv.Chain(p)
    assert c.mark(1) == 0 and c.drain() == []           # ready, but waits for unit 0
    assert c.mark(1) == -3
    assert c.mark(0) == 0 and c.drain() == []
    assert c.mark(7) == -2
    assert c.pending_keys == 2 and c.next_unit == 0
    assert c.mark(2) == 0 and c.drain() == [(0, 2)]
    # next iteration may start on a unit that already ran while others are pending
    assert c.mark(0) == 0 and c.mark(2) == 0
    assert c.drain() == [(0, 1)] and c.next_unit == 1
    assert c.mark(0) == 0 and c.drain() == []           # unit 0 of the following iteration: accepted, waits
    assert c.mark(2) == 0 and c.mark(1) == 0
    assert c.drain() == [(1, 1), (0, 1)]                # finishes the iteration, then wraps


@pytest.mark.skipif(__import__("torch").cuda.is_available(), reason="checks the no-GPU failure path")
def test_init_fails_loudly_without_a_gpu():
    with pytest.raises(kv.KVError) as e:
        kv.KVStore([10, 20], 2, lr=0.1, stream=0)
    assert e.value.status == -6


def test_headers_are_valid_c_and_cxx(tmp_path):
    """The boundary is a C ABI: both headers must compile as C99 and as C++ on their own."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("needs gcc")
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "use_headers.c"
    src.write_text('#include "kv.h"\n#include "kv_engine.h"\n'
                   "int use(kv_store* s, const void* const* g) { kv_sgd_params p = {0.1f, 0.9f, 1e-4f, 0.0f, KV_REDUCE_SEQUENTIAL};\n"
                   "  (void)p; return kv_push(s, 0, g) + kv_wait(s, -1) + KV_SCHED_FUNNEL + KV_FLAG_DESCENDING; }\n")
    for cmd in (["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only"],
                ["g++", "-std=c++17", "-x", "c++", "-Wall", "-Wextra", "-Werror", "-fsyntax-only"]):
        r = subprocess.run(cmd + ["-I", inc, str(src)], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


# ------------------------------------------------------------------ the binding's host-side bounds checks
class _FakeTensor:
    """Carries what the binding looks at before it takes data_ptr()."""

    def __init__(self, numel, dtype="torch.float32", cuda=True, contiguous=True):
        self._n, self.dtype, self.is_cuda, self._c = numel, dtype, cuda, contiguous

    def numel(self):
        return self._n

    def is_contiguous(self):
        return self._c

    def data_ptr(self):
        return 4096


def test_binding_refuses_tensors_that_do_not_match_the_key():
    import torch
    ok = _FakeTensor(100)
    kv.check_tensor(ok, 100, kv.KV_F32, "x")
    for bad, needle in [(_FakeTensor(99), "99 elements"), (_FakeTensor(100, "torch.float16"), "dtype"),
                        (_FakeTensor(100, cuda=False), "GPU memory"), (_FakeTensor(100, contiguous=False), "contiguous"),
                        (torch.zeros(100), "GPU memory")]:
        with pytest.raises(ValueError, match=needle):
            kv.check_tensor(bad, 100, kv.KV_F32, "x")
    with pytest.raises(ValueError, match="dtype"):
        kv.check_tensor(_FakeTensor(100), 100, kv.KV_F16, "x")
    # a push list checks every copy of every key against the key's size and the store's gradient dtype
    numel = [100, 7]
    kv.PushList(2, [0, 1], [[_FakeTensor(100)] * 2, [_FakeTensor(7)] * 2], numel, kv.KV_F32)
    with pytest.raises(ValueError, match="gradient copy 1 of key 1"):
        kv.PushList(2, [0, 1], [[_FakeTensor(100)] * 2, [_FakeTensor(7), _FakeTensor(8)]], numel, kv.KV_F32)
    with pytest.raises(ValueError, match="dtype"):
        kv.PushList(2, [1], [[_FakeTensor(7)] * 2], numel, kv.KV_F16)
    with pytest.raises(ValueError, match="2 gradient copies"):
        kv.PushList(2, [1], [[_FakeTensor(7)]], numel, kv.KV_F32)
