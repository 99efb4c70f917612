"""The five benchmark configurations and a builder for small ad-hoc ones.

Each configuration names a key set, the number W of gradient replicas, the
gradient dtype, the bucket size, the optimizer hyper-parameters and the recipe
for the gradient values.  The paper's workloads are CNN training runs on CIFAR10
and ImageNet-1K (Evaluation section); these synthetic sets stand in for them
with the same tensor shapes and a plausible gradient value distribution.
Bucket sizes are binary units (KiB / MiB).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Sequence

from .keysets import KeySpec, inception_bn_keys, mlp_keys, resnet20_keys, resnet50_keys, vgg16_keys

KIB = 1 << 10
MIB = 1 << 20


@dataclass(frozen=True)
class Config:
    cfg_id: int                 # seed component; 1..5 for the benchmark configs
    name: str
    keys: Sequence[KeySpec]
    W: int
    grad_dtype: str             # "f32" | "f16"
    bucket_bytes: int
    lr: float = 0.1
    momentum: float = 0.9
    wd: float = 1e-4
    sigma_mode: str = "const"   # "const": every key uses sigma_lo; "loguniform": per key in [lo, hi]
    sigma_lo: float = 1e-2
    sigma_hi: float = 1e-2
    zero_frac: float = 0.0      # fraction of keys whose gradients are all zero on every rank

    @property
    def numel(self) -> List[int]:
        return [k.numel for k in self.keys]

    @property
    def total_numel(self) -> int:
        return sum(self.numel)

    @property
    def grad_itemsize(self) -> int:
        return 4 if self.grad_dtype == "f32" else 2

    @property
    def algorithmic_bytes_per_step(self) -> int:
        """W gradient reads + read of w, m + write of w', m' per element."""
        return self.total_numel * (self.W * self.grad_itemsize + 16)


def _cfg1() -> Config:
    return Config(1, "mlp_w2", mlp_keys(), 2, "f32", 64 * KIB,
                  sigma_mode="const", sigma_lo=1e-2, sigma_hi=1e-2)


def _cfg2() -> Config:
    return Config(2, "resnet20_w8", resnet20_keys(), 8, "f32", 256 * KIB,
                  sigma_mode="loguniform", sigma_lo=1e-4, sigma_hi=1e-2)


def _cfg3() -> Config:
    return Config(3, "resnet50_w8", resnet50_keys(), 8, "f32", 4 * MIB,
                  sigma_mode="loguniform", sigma_lo=1e-4, sigma_hi=1e-2, zero_frac=0.05)


def _cfg4() -> Config:
    return Config(4, "resnet50_w32_f16", resnet50_keys(), 32, "f16", 8 * MIB,
                  sigma_mode="loguniform", sigma_lo=1e-4, sigma_hi=1e-2)


def _cfg5() -> Config:
    return Config(5, "vgg16_w16", vgg16_keys(), 16, "f32", 16 * MIB,
                  sigma_mode="const", sigma_lo=1e-3, sigma_hi=1e-3)


def _cfg6() -> Config:
    """The paper's other ImageNet model, with the learning rate it uses at 256 GPUs."""
    return Config(6, "inception_bn_w8", inception_bn_keys(), 8, "f32", 4 * MIB, lr=1.0,
                  sigma_mode="loguniform", sigma_lo=1e-4, sigma_hi=1e-2)


CONFIGS: Dict[int, Callable[[], Config]] = {1: _cfg1, 2: _cfg2, 3: _cfg3, 4: _cfg4, 5: _cfg5, 6: _cfg6}


def scaled_lr(n_gpus: int, base_lr: float = 0.1, lr_at_256: float = 1.0) -> float:
    """Learning rate grown linearly with the number of GPUs (the global mini-batch), through the two
    points the paper states: 0.1 by default and 1.0 at 256 GPUs.  Never below the default."""
    return max(base_lr, lr_at_256 * n_gpus / 256.0)


def get_config(cfg_id: int) -> Config:
    return CONFIGS[cfg_id]()


def tiny_config(numel: Sequence[int], W: int, grad_dtype: str = "f32", bucket_bytes: int = 4 * KIB,
                cfg_id: int = 100, **kw) -> Config:
    """A small configuration with arbitrary key lengths (for tests)."""
    keys = [KeySpec(f"k{i}", (int(n),), "weight", max(int(n), 1)) for i, n in enumerate(numel)]
    return Config(cfg_id, f"tiny{cfg_id}", keys, W, grad_dtype, bucket_bytes, **kw)
