"""Seeded value generators for gradients and initial weights.

Every array is drawn from its own generator seeded by
(config id, step, key, rank), so the values do not depend on the order in
which keys or ranks are generated, on threading, or on the device.  Replicas
get independent draws, not copies.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from typing import List, Optional, Set

import numpy as np

from .configs import Config

_TAG_SIGMA = 0x51674D41
_TAG_ZERO = 0x5A45524F
_TAG_WEIGHT = 0x57454947


def _rng(*seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.SFC64(list(seed)))


def key_sigma(cfg: Config) -> np.ndarray:
    """Per-key gradient standard deviation (float32)."""
    K = len(cfg.keys)
    if cfg.sigma_mode == "const":
        return np.full(K, cfg.sigma_lo, dtype=np.float32)
    u = _rng(cfg.cfg_id, _TAG_SIGMA).random(K)
    lo, hi = math.log10(cfg.sigma_lo), math.log10(cfg.sigma_hi)
    return np.power(10.0, lo + (hi - lo) * u).astype(np.float32)


def zero_keys(cfg: Config) -> Set[int]:
    """Keys whose gradient is exactly zero on every rank and step."""
    K = len(cfg.keys)
    nz = int(round(cfg.zero_frac * K))
    if nz == 0:
        return set()
    perm = _rng(cfg.cfg_id, _TAG_ZERO).permutation(K)
    return set(int(k) for k in perm[:nz])


def make_gradient(cfg: Config, step: int, key: int, rank: int,
                  sigma: Optional[np.ndarray] = None, zeros: Optional[Set[int]] = None) -> np.ndarray:
    """Gradient of one key on one rank: N(0, sigma_key) in float32, rounded to
    nearest-even float16 when the configuration uses half-precision gradients."""
    n = cfg.keys[key].numel
    np_dtype = np.float32 if cfg.grad_dtype == "f32" else np.float16
    if zeros is None:
        zeros = zero_keys(cfg)
    if key in zeros:
        return np.zeros(n, dtype=np_dtype)
    if sigma is None:
        sigma = key_sigma(cfg)
    g = _rng(cfg.cfg_id, step, key, rank).standard_normal(n, dtype=np.float32)
    g *= sigma[key]
    return g if cfg.grad_dtype == "f32" else g.astype(np.float16)


def make_gradients_for_key(cfg: Config, step: int, key: int, threads: int = 1) -> List[np.ndarray]:
    sigma, zeros = key_sigma(cfg), zero_keys(cfg)
    if threads <= 1:
        return [make_gradient(cfg, step, key, r, sigma, zeros) for r in range(cfg.W)]
    with ThreadPoolExecutor(threads) as ex:
        return list(ex.map(lambda r: make_gradient(cfg, step, key, r, sigma, zeros), range(cfg.W)))


def make_step_gradients(cfg: Config, step: int, threads: int = 8) -> List[List[np.ndarray]]:
    """All gradients of one step: result[key][rank]."""
    sigma, zeros = key_sigma(cfg), zero_keys(cfg)
    jobs = [(k, r) for k in range(len(cfg.keys)) for r in range(cfg.W)]
    with ThreadPoolExecutor(max(1, threads)) as ex:
        flat = list(ex.map(lambda kr: make_gradient(cfg, step, kr[0], kr[1], sigma, zeros), jobs))
    W = cfg.W
    return [flat[k * W:(k + 1) * W] for k in range(len(cfg.keys))]


def make_weight(cfg: Config, key: int) -> np.ndarray:
    """Initial value of one key: N(0, 2/fan_in) for matrices and conv kernels,
    one for BN scales, zero for BN shifts and biases."""
    spec = cfg.keys[key]
    n = spec.numel
    if spec.kind == "gamma":
        return np.ones(n, dtype=np.float32)
    if spec.kind in ("beta", "bias"):
        return np.zeros(n, dtype=np.float32)
    w = _rng(cfg.cfg_id, _TAG_WEIGHT, key).standard_normal(n, dtype=np.float32)
    w *= np.float32(math.sqrt(2.0 / max(spec.fan_in, 1)))
    return w


def make_weights(cfg: Config, threads: int = 8) -> List[np.ndarray]:
    with ThreadPoolExecutor(max(1, threads)) as ex:
        return list(ex.map(lambda k: make_weight(cfg, k), range(len(cfg.keys))))
