"""MI355X-native per-key gradient aggregation + SGD update behind a KVStore
push / pull interface (one GPU's share of the paper's data-parallel hot path).

The package is a thin ctypes binding over libkv_mi355x.so (HIP kernels and a C
ABI, declared in include/kv.h).  There is no CPU fallback: importing
``KVStore`` without the built library raises.
"""
from .kvstore import (  # noqa: F401
    KVError, KVStore, Plan, Chain, PushList, check_tensor, load_library, library_path, copy_bytes, read_bytes, stream_mix, evict_caches, null_launch,
    KV_F32, KV_F16, KV_REDUCE_SEQUENTIAL, KV_REDUCE_PAIRWISE, KV_FLAG_KEEP_SUM, KV_FLAG_DESCENDING, KV_FLAG_LAZY_LAUNCH, KV_FLAG_AUTOTUNE, STATUS,
    KV_SCHED_CHAINED, KV_SCHED_FUNNEL, KV_SCHED_CONCURRENT,
)
