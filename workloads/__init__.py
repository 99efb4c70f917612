"""Seeded synthetic inputs: key sets and gradient / weight values.

This package holds no arithmetic of the aggregation method itself (no sums
over replicas, no optimizer update, no bucket packing).  It only produces
tensor shapes and random values, so that the CPU oracle and the HIP path can be
fed identical bits without sharing any other code.
"""
from .keysets import KeySpec, mlp_keys, resnet20_keys, resnet50_keys, vgg16_keys, inception_bn_keys
from .configs import Config, CONFIGS, get_config, tiny_config, scaled_lr
from .generate import (
    key_sigma,
    zero_keys,
    make_gradient,
    make_gradients_for_key,
    make_step_gradients,
    make_weight,
    make_weights,
)

__all__ = [
    "KeySpec", "mlp_keys", "resnet20_keys", "resnet50_keys", "vgg16_keys", "inception_bn_keys", "scaled_lr",
    "Config", "CONFIGS", "get_config", "tiny_config",
    "key_sigma", "zero_keys", "make_gradient", "make_gradients_for_key", "make_step_gradients",
    "make_weight", "make_weights",
]
