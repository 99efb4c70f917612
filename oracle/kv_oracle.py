"""Python face of the CPU oracle.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module; the GPU library never does, and this module imports nothing of it.

* ``OracleStore`` is the key-value store of the paper's KVStore API section
  reduced to its values: ``push`` of the W gradient copies of every key
  aggregates them (sum over ranks), the sum is multiplied by ``rescale``
  (Parallel SGD section) and the weights are updated (eq. (1), extended by
  momentum and weight decay as described in ``kv_oracle.c``).  The loop over keys
  is here, in ascending key order; the loops over ranks and elements are the C
  functions in ``kv_oracle.c``.
* ``plan_units`` is the bucket-packing policy written out as a plain scan.
"""
from __future__ import annotations

import ctypes
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

from . import build as _build

SEQUENTIAL = 0
PAIRWISE = 1
F32 = 0
F16 = 1

_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        # KVO_LIBRARY names another build of kv_oracle.c to load instead: the mutation tests point it
        # at copies with a planted mistake to show that the pins notice.
        path = os.environ.get("KVO_LIBRARY") or _build.build(force=False)
        L = ctypes.CDLL(path)
        vpp = ctypes.POINTER(ctypes.c_void_p)
        fp = ctypes.POINTER(ctypes.c_float)
        L.kvo_half_to_float.restype = ctypes.c_float
        L.kvo_half_to_float.argtypes = [ctypes.c_uint16]
        L.kvo_round_to_half.restype = None
        L.kvo_round_to_half.argtypes = [fp, ctypes.c_int64, ctypes.POINTER(ctypes.c_uint16)]
        L.kvo_reduce_key.restype = ctypes.c_int
        L.kvo_reduce_key.argtypes = [vpp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_int64, ctypes.c_int64, fp]
        L.kvo_step_key.restype = ctypes.c_int
        L.kvo_step_key.argtypes = [vpp, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                   ctypes.c_float, ctypes.c_float, ctypes.c_float, ctypes.c_float,
                                   fp, fp, fp, ctypes.c_int64, ctypes.c_int64]
        _lib = L
    return _lib


def _fptr(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.POINTER(ctypes.c_float)()
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _check_grads(grads: Sequence[np.ndarray]):
    W = len(grads)
    if W < 1:
        raise ValueError("need at least one gradient copy")
    dt = grads[0].dtype
    if dt == np.float32:
        code = F32
    elif dt == np.float16:
        code = F16
    else:
        raise TypeError(f"gradient dtype {dt} not supported")
    n = grads[0].size
    for g in grads:
        if g.dtype != dt or g.size != n or not g.flags.c_contiguous:
            raise ValueError("gradient copies must share dtype and size and be contiguous")
    ptrs = (ctypes.c_void_p * W)(*[g.ctypes.data for g in grads])
    return ptrs, code, W, n


def half_to_float(bits: int) -> float:
    return float(lib().kvo_half_to_float(bits & 0xFFFF))


def round_to_half(x: np.ndarray) -> np.ndarray:
    """binary32 -> binary16, round to nearest even (the value the fp16 replicas of the weights receive)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.size, dtype=np.uint16)
    lib().kvo_round_to_half(_fptr(x), x.size, out.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)))
    return out.view(np.float16).reshape(x.shape)


def reduce_key(grads: Sequence[np.ndarray], order: int = SEQUENTIAL) -> np.ndarray:
    """Raw fp32 sum over the W copies of one key (what the paper's pull returns)."""
    ptrs, code, W, n = _check_grads(grads)
    out = np.empty(n, dtype=np.float32)
    rc = lib().kvo_reduce_key(ptrs, code, W, order, 0, n, _fptr(out))
    if rc != 0:
        raise ValueError("kvo_reduce_key rejected its arguments")
    return out


def step_key(grads: Sequence[np.ndarray], w: np.ndarray, m: np.ndarray, *, rescale: float, lr: float,
             momentum: float, wd: float, order: int = SEQUENTIAL, sum_out: Optional[np.ndarray] = None,
             lo: int = 0, hi: Optional[int] = None) -> None:
    """Aggregate + scale + update one key in place over elements [lo, hi)."""
    ptrs, code, W, n = _check_grads(grads)
    for a in (w, m) + ((sum_out,) if sum_out is not None else ()):
        if a.dtype != np.float32 or a.size != n or not a.flags.c_contiguous:
            raise ValueError("w, m and sum_out must be contiguous float32 of the key's size")
    if hi is None:
        hi = n
    rc = lib().kvo_step_key(ptrs, code, W, order, rescale, lr, momentum, wd,
                            _fptr(w), _fptr(m), _fptr(sum_out), lo, hi)
    if rc != 0:
        raise ValueError("kvo_step_key rejected its arguments")


class OracleStore:
    """Weights and momentum of every key on the host, stepped by the C loops."""

    def __init__(self, numel: Sequence[int], W: int, *, lr: float, momentum: float, wd: float,
                 rescale: Optional[float] = None, order: int = SEQUENTIAL, keep_sum: bool = False):
        self.numel = [int(n) for n in numel]
        self.W = int(W)
        self.lr = float(lr)
        self.momentum = float(momentum)
        self.wd = float(wd)
        # default scale 1/W, rounded once to fp32 and then multiplied
        self.rescale = float(np.float32(1.0) / np.float32(W)) if rescale is None or rescale <= 0 else float(rescale)
        self.order = order
        self.w = [np.zeros(n, dtype=np.float32) for n in self.numel]
        self.m = [np.zeros(n, dtype=np.float32) for n in self.numel]
        self.s = [np.zeros(n, dtype=np.float32) for n in self.numel] if keep_sum else None

    def set_weights(self, key: int, value: np.ndarray) -> None:
        self.w[key][...] = np.asarray(value, dtype=np.float32).reshape(-1)

    def set_momentum(self, key: int, value: np.ndarray) -> None:
        self.m[key][...] = np.asarray(value, dtype=np.float32).reshape(-1)

    def step_one_key(self, key: int, grads: Sequence[np.ndarray], threads: int = 1) -> None:
        n = self.numel[key]
        if len(grads) != self.W:
            raise ValueError("wrong number of gradient copies")
        if n == 0:
            return
        kw = dict(rescale=self.rescale, lr=self.lr, momentum=self.momentum, wd=self.wd, order=self.order,
                  sum_out=None if self.s is None else self.s[key])
        if threads <= 1 or n < 4096 * threads:
            step_key(grads, self.w[key], self.m[key], **kw)
            return
        # the same function on disjoint element ranges: per-element arithmetic is untouched
        edges = [n * t // threads for t in range(threads + 1)]
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(lambda t: step_key(grads, self.w[key], self.m[key], lo=edges[t], hi=edges[t + 1], **kw),
                        range(threads)))

    def step(self, grads: Sequence[Sequence[np.ndarray]], threads: int = 1) -> None:
        """grads[key][rank]; keys are processed in ascending key order."""
        if len(grads) != len(self.numel):
            raise ValueError("one gradient list per key expected")
        for key in range(len(self.numel)):
            self.step_one_key(key, grads[key], threads)


# --------------------------------------------------------------------------
# Bucket packing policy, written as a plain scan over the keys.
# --------------------------------------------------------------------------

@dataclass
class Unit:
    keys: List[int]
    large: bool


def plan_units(numel: Sequence[int], grad_itemsize: int, bucket_bytes: int) -> List[Unit]:
    """Scan keys in ascending id.  A key's size is numel * itemsize of ONE
    gradient copy.  size >= bucket_bytes: the key is a unit of its own and does
    not close the open bucket.  Otherwise it joins the open bucket if the
    bucket's bytes stay <= bucket_bytes, else the bucket is closed and a new one
    opened with this key.  Units are numbered by the id of their first key."""
    units: List[Unit] = []
    open_unit: Optional[Unit] = None
    open_bytes = 0
    for k, n in enumerate(numel):
        size = int(n) * grad_itemsize
        if size >= bucket_bytes:
            units.append(Unit([k], True))
            continue
        if open_unit is not None and open_bytes + size <= bucket_bytes:
            open_unit.keys.append(k)
            open_bytes += size
        else:
            open_unit = Unit([k], False)
            open_bytes = size
            units.append(open_unit)
    units.sort(key=lambda u: u.keys[0])
    return units


def arena_offsets(numel: Sequence[int], units: Sequence[Unit], align_elems: int = 64) -> List[int]:
    """Element offset of every key in the weight / momentum arena: units in
    index order, keys ascending inside a unit, each key start rounded up to a
    multiple of align_elems (256 bytes of fp32: two 128-byte lines of the GPU's
    caches; a layout, no arithmetic of the method depends on it)."""
    off = [0] * len(numel)
    cur = 0
    for u in units:
        for k in u.keys:
            cur = (cur + align_elems - 1) // align_elems * align_elems
            off[k] = cur
            cur += int(numel[k])
    return off
