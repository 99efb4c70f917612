"""The paper's "Dependency Chaining" training-loop listing expressed on the
dependency engine: stand-ins for the backward operators mutate the gradient
variables (last layer first), every push reads its gradient's variable and
mutates the store's variable, which plays the role of the paper's dummy tensor.
Only argument marshalling happens here; the operations themselves are the native
callbacks kv_op_copy and kv_op_push."""
from __future__ import annotations

import ctypes
from typing import List, Sequence

from .engine import CopyArgs, Engine, PushArgs, event_create, event_destroy
from .kvstore import KVError, KVStore


class EngineLoop:
    def __init__(self, store: KVStore, engine: Engine, staged: Sequence, live: Sequence, producer_stream: int,
                 spin: Sequence[int], max_workgroups: int = 0, copy_bytes_cap: int = 0):
        """staged[k], live[k]: device tensors of shape [W, numel_k] (contiguous); the producer of key k
        copies staged[k] to live[k] on producer_stream after spin[k] multiply-adds per lane; the store
        reads rank r of key k at live[k][r].  max_workgroups caps every producer's grid (0 = it fills the
        chip); copy_bytes_cap > 0 makes a producer copy only that many leading bytes, i.e. spend nearly all
        of its time computing (live must then hold valid gradients already)."""
        self.store, self.engine = store, engine
        K = len(live)
        self.K = K
        self.g_var = [engine.new_var() for _ in range(K)]
        self.store_var = engine.new_var()
        self.events = [event_create() for _ in range(K)]
        self.copy_args: List[CopyArgs] = []
        self.push_args: List[PushArgs] = []
        self._keep = [staged, live]
        W = store.W
        for k in range(K):
            nbytes = live[k].numel() * live[k].element_size()
            if copy_bytes_cap > 0:
                nbytes = min(nbytes, copy_bytes_cap) // 16 * 16
            self.copy_args.append(CopyArgs(live[k].data_ptr(), staged[k].data_ptr(), nbytes, producer_stream,
                                           self.events[k], int(spin[k]), 0, int(max_workgroups)))
            ptrs = (ctypes.c_void_p * W)(*[live[k][r].data_ptr() for r in range(W)])
            evs = (ctypes.c_void_p * 1)(self.events[k])
            self._keep += [ptrs, evs]
            self.push_args.append(PushArgs(store._h, k, ptrs, evs, 1, 0))
        # the argument arrays of every kv_engine_push of a step, marshalled once
        c_int, c_vp = ctypes.c_int, ctypes.c_void_p
        self._program = []
        for k in range(K - 1, -1, -1):
            self._program.append((c_vp(engine.op_copy), ctypes.cast(ctypes.pointer(self.copy_args[k]), c_vp),
                                  (c_int * 1)(), 0, (c_int * 1)(self.g_var[k]), 1))
        for k in range(K - 1, -1, -1):
            self._program.append((c_vp(engine.op_push), ctypes.cast(ctypes.pointer(self.push_args[k]), c_vp),
                                  (c_int * 1)(self.g_var[k]), 1, (c_int * 1)(self.store_var), 1))

    def backward_only(self) -> None:
        """Issues the producers directly, last key first (no engine, no pushes)."""
        L = self.engine._L
        for k in range(self.K - 1, -1, -1):
            L.kv_op_copy(ctypes.byref(self.copy_args[k]))

    def step(self) -> None:
        """One iteration: producers, then pushes, all through the engine; returns when every
        operation has been issued to the GPU (not when the GPU is done)."""
        e = self.engine
        push, h = e._L.kv_engine_push, e._h
        for fn, arg, reads, nr, muts, nm in self._program:
            rc = push(h, fn, arg, reads, nr, muts, nm)
            if rc != 0:
                raise KVError(rc, "kv_engine_push")
        e.wait_all()
        for a in self.copy_args:
            if a.status != 0:
                raise KVError(a.status, "producer operation failed")
        for a in self.push_args:
            if a.status != 0:
                raise KVError(a.status, self.store.last_error())

    def close(self) -> None:
        for ev in self.events:
            event_destroy(ev)
        self.events = []
