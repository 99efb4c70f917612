"""ctypes binding of include/kv_engine.h: the minimal dependency engine and its
ready-made GPU operations.  Argument marshalling only."""
from __future__ import annotations

import ctypes
from typing import Callable, List, Optional, Sequence

from .kvstore import KVError, load_library

_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p)
_sigs_done = False


class CopyArgs(ctypes.Structure):
    """kv_op_copy_args"""
    _fields_ = [("dev_dst", ctypes.c_void_p), ("dev_src", ctypes.c_void_p), ("bytes", ctypes.c_size_t),
                ("hip_stream", ctypes.c_void_p), ("record_event", ctypes.c_void_p), ("spin", ctypes.c_int),
                ("status", ctypes.c_int), ("max_workgroups", ctypes.c_int)]


class PushArgs(ctypes.Structure):
    """kv_op_push_args"""
    _fields_ = [("store", ctypes.c_void_p), ("key", ctypes.c_int), ("dev_grads", ctypes.POINTER(ctypes.c_void_p)),
                ("wait_events", ctypes.POINTER(ctypes.c_void_p)), ("n_events", ctypes.c_int), ("status", ctypes.c_int)]


def _lib():
    global _sigs_done
    L = load_library()
    if not _sigs_done:
        c_int, c_vp, P = ctypes.c_int, ctypes.c_void_p, ctypes.POINTER
        L.kv_engine_create.restype = c_int
        L.kv_engine_create.argtypes = [P(c_vp), c_int]
        L.kv_engine_destroy.restype = None
        L.kv_engine_destroy.argtypes = [c_vp]
        L.kv_engine_new_var.restype = c_int
        L.kv_engine_new_var.argtypes = [c_vp, P(c_int)]
        L.kv_engine_push.restype = c_int
        L.kv_engine_push.argtypes = [c_vp, c_vp, c_vp, P(c_int), c_int, P(c_int), c_int]
        L.kv_engine_wait_var.restype = c_int
        L.kv_engine_wait_var.argtypes = [c_vp, c_int]
        L.kv_engine_wait_all.restype = c_int
        L.kv_engine_wait_all.argtypes = [c_vp]
        L.kv_engine_stats.restype = c_int
        L.kv_engine_stats.argtypes = [c_vp, P(ctypes.c_int64), P(c_int)]
        L.kv_event_create.restype = c_int
        L.kv_event_create.argtypes = [P(c_vp)]
        L.kv_event_destroy.restype = None
        L.kv_event_destroy.argtypes = [c_vp]
        L.kv_wait_event.restype = c_int
        L.kv_wait_event.argtypes = [c_vp, c_vp]
        _sigs_done = True
    return L


class Engine:
    """kv_engine_*.  push() takes a Python callable (wrapped as a C callback; it runs on a
    worker thread) or the address of a C function together with the address of its argument."""

    def __init__(self, n_threads: int = 4):
        self._L = _lib()
        h = ctypes.c_void_p()
        rc = self._L.kv_engine_create(ctypes.byref(h), n_threads)
        if rc != 0:
            raise KVError(rc, "kv_engine_create")
        self._h = h
        self._keep: List[object] = []      # callbacks and arguments of operations that may not have run yet
        self._pushed = 0
        self.op_copy = ctypes.cast(self._L.kv_op_copy, ctypes.c_void_p).value
        self.op_push = ctypes.cast(self._L.kv_op_push, ctypes.c_void_p).value

    def close(self) -> None:
        if self._h is not None:
            self._L.kv_engine_destroy(self._h)
            self._h = None
            self._keep.clear()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def new_var(self) -> int:
        v = ctypes.c_int()
        rc = self._L.kv_engine_new_var(self._h, ctypes.byref(v))
        if rc != 0:
            raise KVError(rc, "kv_engine_new_var")
        return v.value

    def push(self, fn, arg=None, read: Sequence[int] = (), mutate: Sequence[int] = ()) -> None:
        if callable(fn):
            cb = _FN(lambda _arg, _f=fn: _f())
            self._keep.append(cb)
            fn_ptr, arg_ptr = ctypes.cast(cb, ctypes.c_void_p), None
        else:
            fn_ptr = ctypes.c_void_p(int(fn))
            if arg is not None:
                self._keep.append(arg)
            arg_ptr = ctypes.cast(ctypes.pointer(arg), ctypes.c_void_p) if isinstance(arg, ctypes.Structure) else arg
        r = (ctypes.c_int * max(len(read), 1))(*read)
        m = (ctypes.c_int * max(len(mutate), 1))(*mutate)
        rc = self._L.kv_engine_push(self._h, fn_ptr, arg_ptr, r, len(read), m, len(mutate))
        if rc != 0:
            raise KVError(rc, "kv_engine_push")
        self._pushed += 1

    def wait_var(self, var: int) -> None:
        rc = self._L.kv_engine_wait_var(self._h, var)
        if rc != 0:
            raise KVError(rc, "kv_engine_wait_var")
        # a loop that only ever waits for single variables must not keep every callback it ever pushed: once the
        # engine has run everything pushed so far (counted after each operation has returned) nothing is referenced
        if self.stats()[0] == self._pushed:
            self._keep.clear()

    def wait_all(self) -> None:
        rc = self._L.kv_engine_wait_all(self._h)
        if rc != 0:
            raise KVError(rc, "kv_engine_wait_all")
        self._keep.clear()

    def stats(self):
        n, mx = ctypes.c_int64(), ctypes.c_int()
        self._L.kv_engine_stats(self._h, ctypes.byref(n), ctypes.byref(mx))
        return n.value, mx.value


def event_create() -> int:
    L = _lib()
    ev = ctypes.c_void_p()
    rc = L.kv_event_create(ctypes.byref(ev))
    if rc != 0:
        raise KVError(rc, "kv_event_create")
    return int(ev.value)


def event_destroy(ev: int) -> None:
    _lib().kv_event_destroy(ctypes.c_void_p(ev))
