"""Shared test helpers: golden-file reader, comparison metric, and a numpy
float32 evaluation of the step used as a cross-check (numpy never contracts
a*b+c into one rounding)."""
from __future__ import annotations

import os
from typing import Dict, List, Sequence

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load_hand_cases(path: str = os.path.join(GOLDEN, "hand_cases.txt")) -> List[Dict]:
    cases: List[Dict] = []
    cur = None
    with open(path) as f:
        for raw in f:
            line = raw.split("#", 1)[0].strip()
            if not line:
                continue
            tok = line.split()
            head, rest = tok[0], tok[1:]
            if head == "case":
                cur = {"name": rest[0], "g": []}
                cases.append(cur)
            elif head == "g":
                cur["g"].append([float(x) for x in rest])
            elif head in ("w", "m", "expect_s", "expect_w", "expect_m"):
                cur[head] = [float(x) for x in rest]
            elif head == "dtype":
                cur["dtype"] = rest[0]
            elif head == "order":
                cur["order"] = int(rest[0])
            else:
                cur[head] = float(rest[0])
    return cases


def within_tol(a: np.ndarray, b: np.ndarray, tol: float) -> bool:
    """|a-b| <= tol * max(|b|, 1e-3 * rms(b)) for every element (b is the reference)."""
    a64 = np.asarray(a, dtype=np.float64)
    b64 = np.asarray(b, dtype=np.float64)
    if a64.size == 0:
        return True
    rms = float(np.sqrt(np.mean(b64 * b64)))
    bound = tol * np.maximum(np.abs(b64), 1e-3 * rms)
    return bool(np.all(np.abs(a64 - b64) <= bound))


def bits_equal(a: np.ndarray, b: np.ndarray) -> bool:
    a = np.ascontiguousarray(a, dtype=np.float32)
    b = np.ascontiguousarray(b, dtype=np.float32)
    return a.shape == b.shape and bool(np.array_equal(a.view(np.uint32), b.view(np.uint32)))


def max_ulp(a: np.ndarray, b: np.ndarray) -> int:
    def key(x):
        i = np.ascontiguousarray(x, dtype=np.float32).view(np.int32).astype(np.int64)
        return np.where(i < 0, -(i & 0x7FFFFFFF), i)
    if np.asarray(a).size == 0:
        return 0
    return int(np.max(np.abs(key(a) - key(b))))


def numpy_fold(grads: Sequence[np.ndarray], order: int) -> np.ndarray:
    v = [np.asarray(g).astype(np.float32) for g in grads]

    def tree(lo, n):
        if n == 1:
            return v[lo]
        h = 1
        while 2 * h < n:
            h *= 2
        return tree(lo, h) + tree(lo + h, n - h)

    if order == 1:
        return tree(0, len(v))
    s = v[0].copy()
    for r in range(1, len(v)):
        s = s + v[r]
    return s


def numpy_step(grads, w, m, *, rescale, lr, momentum, wd, order=0):
    """Vectorised float32 evaluation; returns (s, w', m')."""
    f = np.float32
    s = numpy_fold(grads, order)
    ghat = f(rescale) * s
    t = ghat + f(wd) * w
    dw = f(momentum) * m - f(lr) * t
    return s, (w + dw).astype(np.float32), dw.astype(np.float32)
