"""ctypes binding of include/kv.h: argument marshalling only.

Names follow the C ABI (kv_init -> KVStore(...), kv_push -> KVStore.push, ...).
Tensors are torch tensors on the GPU; only their ``data_ptr()`` crosses the
boundary.  PyTorch supplies device memory and the stream, nothing else.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

KV_F32, KV_F16 = 0, 1
KV_REDUCE_SEQUENTIAL, KV_REDUCE_PAIRWISE = 0, 1
KV_FLAG_KEEP_SUM = 1
KV_FLAG_DESCENDING = 2
KV_FLAG_LAZY_LAUNCH = 4
KV_FLAG_AUTOTUNE = 8
KV_SCHED_CHAINED, KV_SCHED_FUNNEL, KV_SCHED_CONCURRENT = 0, 1, 2
STATUS = {0: "KV_OK", -1: "KV_ERR_ARG", -2: "KV_ERR_KEY", -3: "KV_ERR_STATE", -4: "KV_ERR_ALIGN",
          -5: "KV_ERR_INCOMPLETE", -6: "KV_ERR_HIP", -7: "KV_ERR_NOMEM"}

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libkv_mi355x.so")
_lib: Optional[ctypes.CDLL] = None


class KVError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS.get(status, status)}: {message}")
        self.status = status


class _SgdParams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("momentum", ctypes.c_float), ("wd", ctypes.c_float),
                ("rescale", ctypes.c_float), ("reduce_order", ctypes.c_int)]


class _Tuning(ctypes.Structure):
    _fields_ = [("unroll", ctypes.c_int), ("workgroups_per_cu", ctypes.c_int), ("nontemporal", ctypes.c_int),
                ("xcd_remap", ctypes.c_int), ("lane_elems", ctypes.c_int), ("resident_workgroups", ctypes.c_int),
                ("run_time_w", ctypes.c_int)]


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Loads the built library.  It is never built or replaced by a fallback here."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_1802_06949_amd.build`")
    L = ctypes.CDLL(_LIB_PATH)
    c_int, c_i64, c_vp, c_sz = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    P = ctypes.POINTER

    def sig(name, res, *args):
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = list(args)

    sig("kv_plan_create", c_int, P(c_vp), c_int, P(c_i64), c_int, c_sz)
    sig("kv_plan_destroy", None, c_vp)
    sig("kv_plan_num_keys", c_int, c_vp)
    sig("kv_plan_num_units", c_int, c_vp)
    sig("kv_plan_unit", c_int, c_vp, c_int, P(c_int), P(c_int), P(c_int), c_int)
    sig("kv_plan_key", c_int, c_vp, c_int, P(c_int), P(c_i64))
    sig("kv_plan_arena_numel", c_i64, c_vp)
    sig("kv_chain_create", c_int, P(c_vp), c_vp)
    sig("kv_chain_destroy", None, c_vp)
    sig("kv_chain_set_descending", c_int, c_vp, c_int)
    sig("kv_chain_mark", c_int, c_vp, c_int)
    sig("kv_chain_next_run", c_int, c_vp, P(c_int), P(c_int))
    sig("kv_chain_pending_keys", c_int, c_vp)
    sig("kv_chain_next_unit", c_int, c_vp)
    sig("kv_init", c_int, P(c_vp), c_int, P(c_i64), c_int, c_int, c_sz, P(_SgdParams), ctypes.c_uint, P(_Tuning), c_vp)
    sig("kv_destroy", None, c_vp)
    sig("kv_set_weights", c_int, c_vp, c_int, c_vp)
    sig("kv_set_momentum", c_int, c_vp, c_int, c_vp)
    sig("kv_set_lr", c_int, c_vp, ctypes.c_float)
    sig("kv_set_sgd_params", c_int, c_vp, P(_SgdParams))
    sig("kv_get_sgd_params", c_int, c_vp, P(_SgdParams))
    sig("kv_push", c_int, c_vp, c_int, P(c_vp))
    sig("kv_push_list", c_int, c_vp, c_int, P(c_int), P(c_vp))
    sig("kv_push_list_noalloc", c_int, c_vp, c_int, P(c_int), P(c_vp))
    sig("kv_pull", c_int, c_vp, c_int, c_vp)
    sig("kv_pull_list", c_int, c_vp, c_int, P(c_int), P(c_vp))
    sig("kv_pull_grad", c_int, c_vp, c_int, c_vp)
    sig("kv_pull_momentum", c_int, c_vp, c_int, c_vp)
    sig("kv_weights_ptr", c_int, c_vp, c_int, P(c_vp))
    sig("kv_wait", c_int, c_vp, c_int)
    sig("kv_set_broadcast", c_int, c_vp, c_int, c_int, P(c_vp), c_int)
    sig("kv_set_schedule", c_int, c_vp, c_int, c_int, c_int)
    sig("kv_barrier", c_int, c_vp)
    sig("kv_get_tuning", c_int, c_vp, P(_Tuning), P(c_int))
    sig("kv_wide_launches", c_int, c_vp, P(c_i64))
    sig("kv_broadcast_weights", c_int, c_vp, c_int)
    sig("kv_release_captures", c_int, c_vp)
    sig("kv_store_plan", c_vp, c_vp)
    sig("kv_launch_log", c_int, c_vp, P(c_i64), P(c_int), P(c_int), c_int)
    sig("kv_timing_begin", c_int, c_vp)
    sig("kv_timing_end", c_int, c_vp, P(ctypes.c_float), P(c_i64))
    sig("kv_timing_mark", c_int, c_vp)
    sig("kv_timing_intervals", c_int, c_vp, P(ctypes.c_float), c_int)
    sig("kv_copy_bytes", c_int, c_vp, c_vp, c_sz, c_vp)
    sig("kv_read_bytes", c_int, c_vp, c_sz, c_vp)
    sig("kv_stream_mix", c_int, P(c_vp), c_int, c_int, c_sz, c_vp)
    sig("kv_evict_caches", c_int, c_vp, c_sz, c_int, c_vp)
    sig("kv_null_launch", c_int, c_int, c_vp)
    sig("kv_push_list_repeat", c_int, c_vp, c_int, P(c_int), P(c_vp), c_int)
    sig("kv_completion_events", c_int, c_vp, P(c_i64))
    sig("kv_last_error", ctypes.c_char_p, c_vp)
    _lib = L
    return L


def _dtype_code(grad_dtype) -> int:
    if grad_dtype in (KV_F32, "f32", "float32"):
        return KV_F32
    if grad_dtype in (KV_F16, "f16", "float16"):
        return KV_F16
    raise ValueError(f"unknown gradient dtype {grad_dtype!r}")


def _global_error(L) -> str:
    return L.kv_last_error(None).decode()


class Plan:
    """kv_plan_*: the bucket plan (host only)."""

    def __init__(self, key_numel: Sequence[int], grad_dtype="f32", bucket_bytes: int = 1 << 22, _borrowed=None):
        self._L = load_library()
        self._owned = _borrowed is None
        if _borrowed is not None:
            self._h = ctypes.c_void_p(_borrowed)
            return
        n = len(key_numel)
        arr = (ctypes.c_int64 * max(n, 1))(*[int(x) for x in key_numel])
        h = ctypes.c_void_p()
        rc = self._L.kv_plan_create(ctypes.byref(h), n, arr, _dtype_code(grad_dtype), int(bucket_bytes))
        if rc != 0:
            raise KVError(rc, _global_error(self._L))
        self._h = h

    def __del__(self):
        if getattr(self, "_owned", False) and getattr(self, "_h", None):
            self._L.kv_plan_destroy(self._h)
            self._h = None

    @property
    def num_keys(self) -> int:
        return self._L.kv_plan_num_keys(self._h)

    @property
    def num_units(self) -> int:
        return self._L.kv_plan_num_units(self._h)

    @property
    def arena_numel(self) -> int:
        return self._L.kv_plan_arena_numel(self._h)

    def unit(self, u: int) -> Tuple[List[int], bool]:
        large, nk = ctypes.c_int(), ctypes.c_int()
        rc = self._L.kv_plan_unit(self._h, u, ctypes.byref(large), ctypes.byref(nk), None, 0)
        if rc != 0:
            raise KVError(rc, f"unit {u}")
        keys = (ctypes.c_int * max(nk.value, 1))()
        self._L.kv_plan_unit(self._h, u, None, None, keys, nk.value)
        return list(keys[:nk.value]), bool(large.value)

    def units(self) -> List[Tuple[List[int], bool]]:
        return [self.unit(u) for u in range(self.num_units)]

    def key(self, k: int) -> Tuple[int, int]:
        unit, off = ctypes.c_int(), ctypes.c_int64()
        rc = self._L.kv_plan_key(self._h, k, ctypes.byref(unit), ctypes.byref(off))
        if rc != 0:
            raise KVError(rc, f"key {k}")
        return unit.value, off.value


class Chain:
    """kv_chain_*: the launch-order state machine (host only)."""

    def __init__(self, plan: Plan):
        self._L = load_library()
        self._plan = plan
        h = ctypes.c_void_p()
        rc = self._L.kv_chain_create(ctypes.byref(h), plan._h)
        if rc != 0:
            raise KVError(rc, _global_error(self._L))
        self._h = h

    def __del__(self):
        if getattr(self, "_h", None):
            self._L.kv_chain_destroy(self._h)
            self._h = None

    def set_descending(self, descending: bool) -> int:
        return self._L.kv_chain_set_descending(self._h, 1 if descending else 0)

    def mark(self, key: int) -> int:
        return self._L.kv_chain_mark(self._h, key)

    def next_run(self) -> Optional[Tuple[int, int]]:
        first, n = ctypes.c_int(), ctypes.c_int()
        return (first.value, n.value) if self._L.kv_chain_next_run(self._h, ctypes.byref(first), ctypes.byref(n)) == 1 else None

    def drain(self) -> List[Tuple[int, int]]:
        runs = []
        while True:
            r = self.next_run()
            if r is None:
                return runs
            runs.append(r)

    @property
    def pending_keys(self) -> int:
        return self._L.kv_chain_pending_keys(self._h)

    @property
    def next_unit(self) -> int:
        return self._L.kv_chain_next_unit(self._h)


_TORCH_DTYPE = {KV_F32: "torch.float32", KV_F16: "torch.float16"}


_torch_dtypes = None


def check_tensor(t, numel: int, dtype_code: int, what: str) -> None:
    """Host-side bounds check before a pointer crosses the C ABI: the kernels read or write exactly `numel`
    elements of the given dtype at data_ptr(), so anything else would be an out-of-bounds device access.
    The passing case is four attribute reads (this runs once per gradient copy of every push)."""
    global _torch_dtypes
    if numel == 0:
        return                                       # nothing of an empty key is ever read or written
    if _torch_dtypes is None:
        import torch
        _torch_dtypes = {KV_F32: torch.float32, KV_F16: torch.float16}
    try:
        if t.is_cuda and t.dtype is _torch_dtypes[dtype_code] and t.numel() == numel and t.is_contiguous():
            return
    except AttributeError:
        pass
    if not getattr(t, "is_cuda", False):
        raise ValueError(f"{what}: expected a tensor in GPU memory")
    if str(t.dtype) != _TORCH_DTYPE[dtype_code]:
        raise ValueError(f"{what}: dtype {t.dtype}, expected {_TORCH_DTYPE[dtype_code]}")
    if t.numel() != numel:
        raise ValueError(f"{what}: {t.numel()} elements, the key has {numel}")
    if not t.is_contiguous():
        raise ValueError(f"{what}: tensor is not contiguous")


class PushList:
    """Pre-marshalled arguments of kv_push_list; keeps the tensors alive.  With key_numel and grad_dtype (as
    KVStore.make_push_list passes them) every tensor is checked against its key first."""

    def __init__(self, W: int, keys: Sequence[int], grads: Sequence[Sequence], key_numel: Optional[Sequence[int]] = None,
                 grad_dtype: int = KV_F32):
        if len(keys) != len(grads):
            raise ValueError("one gradient list per key expected")
        self.n = len(keys)
        self.keys = (ctypes.c_int * max(self.n, 1))(*[int(k) for k in keys])
        flat = []
        for key, g in zip(keys, grads):
            if len(g) != W:
                raise ValueError(f"expected {W} gradient copies per key")
            if key_numel is not None and 0 <= int(key) < len(key_numel):      # an unknown key is the library's to refuse
                for r, t in enumerate(g):
                    check_tensor(t, key_numel[int(key)], grad_dtype, f"gradient copy {r} of key {key}")
            flat.extend(int(t.data_ptr()) for t in g)
        self.ptrs = (ctypes.c_void_p * max(len(flat), 1))(*flat)
        self._keep = grads


class KVStore:
    """kv_init ... kv_destroy: one store for a fixed key set (argument marshalling only; see include/kv.h).

    key_numel[k] is the element count of key k; W gradient copies per key of dtype grad_dtype ("f32" / "f16");
    keys smaller than bucket_bytes (one copy) are packed into buckets.  keep_sum / descending / lazy / autotune are
    the kv_flags; stream is a hipStream_t address (default: torch's current stream); the remaining keyword
    arguments are the kv_tuning fields (0 or -1 = the library's default).
    """

    def __init__(self, key_numel: Sequence[int], W: int, grad_dtype="f32", bucket_bytes: int = 1 << 22, *,
                 lr: float, momentum: float = 0.0, wd: float = 0.0, rescale: float = 0.0,
                 reduce_order: int = KV_REDUCE_SEQUENTIAL, keep_sum: bool = False, descending: bool = False, lazy: bool = False,
                 stream: Optional[int] = None,
                 unroll: int = 0, workgroups_per_cu: int = -1, nontemporal: int = -1, xcd_remap: int = -1,
                 lane_elems: int = 0, resident_workgroups: int = 0, run_time_w: int = 0, autotune: bool = False):
        self._L = load_library()
        self._h = None
        self.key_numel = [int(x) for x in key_numel]
        self.W = int(W)
        self.grad_dtype = _dtype_code(grad_dtype)
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        self.stream = int(stream)
        n = len(self.key_numel)
        arr = (ctypes.c_int64 * max(n, 1))(*self.key_numel)
        p = _SgdParams(lr, momentum, wd, rescale, reduce_order)
        t = _Tuning(unroll, workgroups_per_cu, nontemporal, xcd_remap, lane_elems, resident_workgroups, run_time_w)
        h = ctypes.c_void_p()
        rc = self._L.kv_init(ctypes.byref(h), n, arr, self.grad_dtype, self.W, int(bucket_bytes), ctypes.byref(p),
                             (KV_FLAG_KEEP_SUM if keep_sum else 0) | (KV_FLAG_DESCENDING if descending else 0) |
                             (KV_FLAG_LAZY_LAUNCH if lazy else 0) | (KV_FLAG_AUTOTUNE if autotune else 0),
                             ctypes.byref(t), ctypes.c_void_p(self.stream))
        if rc != 0:
            raise KVError(rc, _global_error(self._L))
        self._h = h
        self.plan = Plan([], _borrowed=self._L.kv_store_plan(h))

    def close(self) -> None:
        if self._h is not None:
            self._L.kv_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int) -> None:
        if rc != 0:
            raise KVError(rc, self._L.kv_last_error(self._h).decode())

    # --- values
    def _check_f32(self, key: int, t, what: str) -> None:
        if 0 <= key < len(self.key_numel):                 # an unknown key is the library's to refuse
            check_tensor(t, self.key_numel[key], KV_F32, f"{what} of key {key}")

    def set_weights(self, key: int, src) -> None:
        self._check_f32(key, src, "initial weights")
        self._check(self._L.kv_set_weights(self._h, key, ctypes.c_void_p(src.data_ptr())))

    def set_momentum(self, key: int, src) -> None:
        self._check_f32(key, src, "momentum")
        self._check(self._L.kv_set_momentum(self._h, key, ctypes.c_void_p(src.data_ptr())))

    def set_lr(self, lr: float) -> None:
        self._check(self._L.kv_set_lr(self._h, lr))

    def set_sgd_params(self, *, lr: float, momentum: float, wd: float, rescale: float = 0.0,
                       reduce_order: int = KV_REDUCE_SEQUENTIAL) -> None:
        p = _SgdParams(lr, momentum, wd, rescale, reduce_order)
        self._check(self._L.kv_set_sgd_params(self._h, ctypes.byref(p)))

    def get_sgd_params(self) -> dict:
        p = _SgdParams()
        self._check(self._L.kv_get_sgd_params(self._h, ctypes.byref(p)))
        return dict(lr=p.lr, momentum=p.momentum, wd=p.wd, rescale=p.rescale, reduce_order=p.reduce_order)

    # --- push
    def push(self, key: int, grads: Sequence) -> None:
        if len(grads) != self.W:
            raise ValueError(f"expected {self.W} gradient copies")
        if 0 <= key < len(self.key_numel):
            for r, g in enumerate(grads):
                check_tensor(g, self.key_numel[key], self.grad_dtype, f"gradient copy {r} of key {key}")
        ptrs = (ctypes.c_void_p * self.W)(*[int(g.data_ptr()) for g in grads])
        self._check(self._L.kv_push(self._h, key, ptrs))

    def push_raw(self, key: int, ptrs: Sequence[int]) -> int:
        """kv_push with raw addresses; returns the status instead of raising."""
        arr = (ctypes.c_void_p * max(len(ptrs), 1))(*[int(p) for p in ptrs])
        return self._L.kv_push(self._h, key, arr)

    def make_push_list(self, keys: Sequence[int], grads: Sequence[Sequence]) -> PushList:
        return PushList(self.W, keys, grads, self.key_numel, self.grad_dtype)

    def push_list(self, pl: PushList) -> None:
        self._check(self._L.kv_push_list(self._h, pl.n, pl.keys, pl.ptrs))

    def push_list_repeat(self, pl: PushList, reps: int) -> None:
        """kv_push_list_repeat (kv_diag.h): the same list push `reps` times from native code, for timing
        launch-bound stores without the interpreter between the launches."""
        self._check(self._L.kv_push_list_repeat(self._h, pl.n, pl.keys, pl.ptrs, int(reps)))

    def completion_events(self) -> int:
        """kv_completion_events (kv_diag.h): completion events recorded so far for wait(key)."""
        n = ctypes.c_int64()
        self._check(self._L.kv_completion_events(self._h, ctypes.byref(n)))
        return int(n.value)

    def push_list_noalloc(self, pl: PushList) -> None:
        """kv_push_list_noalloc: the list push that allocates and uploads nothing (static device pointer table)."""
        self._check(self._L.kv_push_list_noalloc(self._h, pl.n, pl.keys, pl.ptrs))

    def get_tuning(self) -> Tuple[dict, bool]:
        """kv_get_tuning: the launch tuning in force and whether a self-tuning store has settled."""
        t, done = _Tuning(), ctypes.c_int()
        self._check(self._L.kv_get_tuning(self._h, ctypes.byref(t), ctypes.byref(done)))
        return {name: getattr(t, name) for name, _ in _Tuning._fields_}, bool(done.value)

    def wide_launches(self) -> int:
        """kv_wide_launches: launches that ran four elements per lane because their gradient buffers are off the
        128-byte line grid."""
        n = ctypes.c_int64()
        self._check(self._L.kv_wide_launches(self._h, ctypes.byref(n)))
        return n.value

    def release_captures(self) -> None:
        """Lets the pointer tables that captured launches read be reused (call once the graphs are gone)."""
        self._check(self._L.kv_release_captures(self._h))

    # --- pull
    def pull(self, key: int, out) -> None:
        self._check_f32(key, out, "pull destination")
        self._check(self._L.kv_pull(self._h, key, ctypes.c_void_p(out.data_ptr())))

    def pull_list(self, keys: Sequence[int], outs: Sequence) -> None:
        n = len(keys)
        if len(outs) != n:
            raise ValueError("one destination per key expected")
        for k, o in zip(keys, outs):
            self._check_f32(int(k), o, "pull destination")
        karr = (ctypes.c_int * max(n, 1))(*[int(k) for k in keys])
        parr = (ctypes.c_void_p * max(n, 1))(*[int(o.data_ptr()) for o in outs])
        self._check(self._L.kv_pull_list(self._h, n, karr, parr))

    def pull_grad(self, key: int, out) -> None:
        self._check_f32(key, out, "pull destination")
        self._check(self._L.kv_pull_grad(self._h, key, ctypes.c_void_p(out.data_ptr())))

    def pull_momentum(self, key: int, out) -> None:
        self._check_f32(key, out, "pull destination")
        self._check(self._L.kv_pull_momentum(self._h, key, ctypes.c_void_p(out.data_ptr())))

    def weights_ptr(self, key: int) -> int:
        p = ctypes.c_void_p()
        self._check(self._L.kv_weights_ptr(self._h, key, ctypes.byref(p)))
        return int(p.value or 0)

    def wait(self, key: int = -1) -> None:
        self._check(self._L.kv_wait(self._h, key))

    def wait_status(self, key: int = -1) -> int:
        return self._L.kv_wait(self._h, key)

    def set_broadcast(self, key: int, replicas: Sequence, dtype="f32") -> None:
        """kv_set_broadcast: replicas is a list of tensors (or raw addresses) that receive the key's new weights."""
        code = _dtype_code(dtype)
        for i, r in enumerate(replicas):
            if not isinstance(r, int) and 0 <= key < len(self.key_numel):
                check_tensor(r, self.key_numel[key], code, f"replica {i} of key {key}")
        ptrs = [int(r) if isinstance(r, int) else int(r.data_ptr()) for r in replicas]
        arr = (ctypes.c_void_p * max(len(ptrs), 1))(*ptrs)
        self._check(self._L.kv_set_broadcast(self._h, key, len(ptrs), arr, _dtype_code(dtype)))
        self._bcast_keep = getattr(self, "_bcast_keep", {})
        self._bcast_keep[key] = replicas

    def broadcast_weights(self, key: int = -1) -> None:
        """kv_broadcast_weights: copies the current weights of a key (-1: all) to its replicas."""
        self._check(self._L.kv_broadcast_weights(self._h, key))

    def set_schedule(self, schedule: int, n_streams: int = 1, outstanding: int = 0) -> None:
        self._check(self._L.kv_set_schedule(self._h, schedule, n_streams, outstanding))

    def barrier(self) -> None:
        self._check(self._L.kv_barrier(self._h))

    # --- introspection
    def launch_log(self, cap: int = 4096) -> Tuple[int, List[Tuple[int, int]]]:
        total = ctypes.c_int64()
        first = (ctypes.c_int * cap)()
        nun = (ctypes.c_int * cap)()
        n = self._L.kv_launch_log(self._h, ctypes.byref(total), first, nun, cap)
        if n < 0:
            raise KVError(n, "kv_launch_log")
        return total.value, [(first[i], nun[i]) for i in range(n)]

    def timing_begin(self) -> None:
        self._check(self._L.kv_timing_begin(self._h))

    def timing_end(self) -> Tuple[float, int]:
        ms, n = ctypes.c_float(), ctypes.c_int64()
        self._check(self._L.kv_timing_end(self._h, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    def timing_mark(self) -> None:
        self._check(self._L.kv_timing_mark(self._h))

    def timing_intervals(self, cap: int = 8192) -> List[float]:
        buf = (ctypes.c_float * cap)()
        n = self._L.kv_timing_intervals(self._h, buf, cap)
        if n < 0:
            raise KVError(n, self.last_error())
        return [buf[i] for i in range(n)]

    def last_error(self) -> str:
        return self._L.kv_last_error(self._h).decode()


def copy_bytes(dst, src, nbytes: int, stream: Optional[int] = None) -> None:
    """kv_copy_bytes: the plain streaming copy kernel used to calibrate byte counters."""
    L = load_library()
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    rc = L.kv_copy_bytes(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()), int(nbytes),
                         ctypes.c_void_p(int(stream)))
    if rc != 0:
        raise KVError(rc, _global_error(L))


def read_bytes(src, nbytes: int, stream: Optional[int] = None) -> None:
    """kv_read_bytes: the plain streaming read kernel (a measured ceiling for reads)."""
    L = load_library()
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    rc = L.kv_read_bytes(ctypes.c_void_p(src.data_ptr()), int(nbytes), ctypes.c_void_p(int(stream)))
    if rc != 0:
        raise KVError(rc, _global_error(L))


def stream_mix(read_bufs: Sequence, write_bufs: Sequence, nbytes: int, stream: Optional[int] = None) -> None:
    """kv_stream_mix: sums 16-byte vectors of the read buffers into every written buffer (a measured ceiling for a
    mix of read and write streams)."""
    L = load_library()
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    bufs = list(read_bufs) + list(write_bufs)
    arr = (ctypes.c_void_p * max(len(bufs), 1))(*[int(b.data_ptr()) for b in bufs])
    rc = L.kv_stream_mix(arr, len(read_bufs), len(write_bufs), int(nbytes), ctypes.c_void_p(int(stream)))
    if rc != 0:
        raise KVError(rc, _global_error(L))


def evict_caches(buf, nbytes: int, dirty: bool = False, stream: Optional[int] = None) -> None:
    """kv_evict_caches: plain cached pass over a scratch buffer (cold-state timing); buf is a tensor or an address."""
    L = load_library()
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    addr = int(buf) if isinstance(buf, int) else buf.data_ptr()
    rc = L.kv_evict_caches(ctypes.c_void_p(addr), int(nbytes), 1 if dirty else 0, ctypes.c_void_p(int(stream)))
    if rc != 0:
        raise KVError(rc, _global_error(L))


def null_launch(count: int = 1, stream: Optional[int] = None) -> None:
    """kv_null_launch: `count` empty kernels back to back (the launch-latency floor)."""
    L = load_library()
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    rc = L.kv_null_launch(int(count), ctypes.c_void_p(int(stream)))
    if rc != 0:
        raise KVError(rc, _global_error(L))
