"""Drives the GPU store and the CPU oracle on the same seeded inputs and compares
them element by element.  Used by the -m gpu tests and by the smoke check."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np

import workloads as wl
from oracle import kv_oracle as orc


def same_bits_or_both_nan(a: np.ndarray, b: np.ndarray) -> bool:
    """Bit equality; NaN payloads are left unspecified (both sides must be NaN)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    if a.shape != b.shape:
        return False
    eq = a.view(np.uint32) == b.view(np.uint32)
    if eq.all():
        return True
    return bool(np.all(eq | (np.isnan(a) & np.isnan(b))))


def first_mismatch(a: np.ndarray, b: np.ndarray) -> str:
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    bad = np.flatnonzero((a.view(np.uint32) != b.view(np.uint32)) & ~(np.isnan(a) & np.isnan(b)))
    if bad.size == 0:
        return "no mismatch"
    i = int(bad[0])
    return f"{bad.size} mismatches, first at {i}: gpu={a[i]!r} ({a.view(np.uint32)[i]:#x}) oracle={b[i]!r} ({b.view(np.uint32)[i]:#x})"


def to_device(arr: np.ndarray, misalign: int = 0):
    """Uploads a host array; with misalign > 0 the data starts that many elements
    into a larger allocation (so its address is not 16-byte aligned)."""
    import torch
    t = torch.from_numpy(arr)
    if misalign == 0:
        return t.cuda()
    buf = torch.empty(arr.size + misalign + 8, dtype=t.dtype, device="cuda")
    view = buf[misalign:misalign + arr.size]
    view.copy_(t)
    return view


class Pair:
    """A GPU store and an oracle store with the same keys and parameters."""

    def __init__(self, numel: Sequence[int], W: int, grad_dtype: str, bucket_bytes: int, *, lr: float, momentum: float,
                 wd: float, rescale: float = 0.0, order: int = 0, keep_sum: bool = True, schedule=None, **tuning):
        import paper_1802_06949_amd as kv
        self.kv = kv
        self.numel = [int(n) for n in numel]
        self.W = W
        self.grad_dtype = grad_dtype
        self.gpu = kv.KVStore(self.numel, W, grad_dtype, bucket_bytes, lr=lr, momentum=momentum, wd=wd, rescale=rescale,
                              reduce_order=order, keep_sum=keep_sum, **tuning)
        self.cpu = orc.OracleStore(self.numel, W, lr=lr, momentum=momentum, wd=wd, rescale=rescale, order=order,
                                   keep_sum=keep_sum)
        self.keep_sum = keep_sum
        if schedule is not None:
            self.gpu.set_schedule(*schedule)

    def set_weights(self, weights: Sequence[np.ndarray]) -> None:
        for k, w in enumerate(weights):
            self.cpu.set_weights(k, w)
            if w.size:
                self.gpu.set_weights(k, to_device(np.ascontiguousarray(w, dtype=np.float32)))
        self.gpu.wait()

    def set_momentum(self, moms: Sequence[np.ndarray]) -> None:
        for k, m in enumerate(moms):
            self.cpu.set_momentum(k, m)
            if m.size:
                self.gpu.set_momentum(k, to_device(np.ascontiguousarray(m, dtype=np.float32)))
        self.gpu.wait()

    def upload(self, grads: Sequence[Sequence[np.ndarray]], misalign: int = 0):
        return [[to_device(g, misalign) for g in gk] for gk in grads]

    def step(self, grads: Sequence[Sequence[np.ndarray]], *, mode: str = "list", order: Optional[Sequence[int]] = None,
             misalign: int = 0, dev=None, oracle_threads: int = 1):
        """mode 'list': one kv_push_list with all keys; 'each': kv_push per key in `order`."""
        K = len(self.numel)
        if dev is None:
            dev = self.upload(grads, misalign)
        keys = list(range(K)) if order is None else list(order)
        if mode == "list":
            pl = self.gpu.make_push_list(keys, [dev[k] for k in keys])
            self.gpu.push_list(pl)
        else:
            for k in keys:
                self.gpu.push(k, dev[k])
        self.gpu.wait()
        self.cpu.step(grads, threads=oracle_threads)
        return dev

    def fetch(self, what: str, key: int) -> np.ndarray:
        import torch
        out = torch.empty(self.numel[key], dtype=torch.float32, device="cuda")
        getattr(self.gpu, {"w": "pull", "m": "pull_momentum", "s": "pull_grad"}[what])(key, out)
        self.gpu.wait()
        return out.cpu().numpy()

    def compare(self, label: str = "") -> None:
        for k in range(len(self.numel)):
            kinds = ("s", "m", "w") if self.keep_sum else ("m", "w")
            for what in kinds:
                got = self.fetch(what, k)
                ref = {"w": self.cpu.w, "m": self.cpu.m, "s": self.cpu.s}[what][k]
                assert same_bits_or_both_nan(got, ref), \
                    f"{label} key {k} ({self.numel[k]} elements) {what}: {first_mismatch(got, ref)}"

    def close(self) -> None:
        self.gpu.close()


def run_config(cfg: wl.Config, steps: int, *, order: int = 0, mode: str = "list", keep_sum: bool = True,
               gen_threads: int = 8, oracle_threads: int = 1, rotate_after_first: bool = False, label: str = "",
               schedule=None, **tuning) -> None:
    """Steps a benchmark configuration on both sides and compares after every step."""
    pair = Pair(cfg.numel, cfg.W, cfg.grad_dtype, cfg.bucket_bytes, lr=cfg.lr, momentum=cfg.momentum, wd=cfg.wd,
                order=order, keep_sum=keep_sum, schedule=schedule, **tuning)
    try:
        pair.set_weights(wl.make_weights(cfg, gen_threads))
        grads = dev = None
        for t in range(steps):
            if t == 0 or not rotate_after_first:
                grads = wl.make_step_gradients(cfg, t, gen_threads)
                dev = None
            else:
                # reuse step 0's values with the ranks rotated by one (cheap fresh-looking step)
                grads = [gk[1:] + gk[:1] for gk in grads]
                dev = [dk[1:] + dk[:1] for dk in dev]
            dev = pair.step(grads, mode=mode, dev=dev, oracle_threads=oracle_threads)
            pair.compare(f"{label or cfg.name} step {t}")
    finally:
        pair.close()
