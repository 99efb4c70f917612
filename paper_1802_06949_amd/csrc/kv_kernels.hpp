// Host-callable launchers of the HIP kernels.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stddef.h>

#include "kv_device.hpp"

// One launcher per (gradient dtype, W) translation unit of kv_fused.hip.
#define KV_DECL_FUSED(F, W) \
    hipError_t kv_launch_fused_f##F##_w##W(const KvKernelSel&, const KvLaunchArgs&, unsigned grid, hipStream_t);
KV_DECL_FUSED(0, 0) KV_DECL_FUSED(0, 2) KV_DECL_FUSED(0, 4) KV_DECL_FUSED(0, 8) KV_DECL_FUSED(0, 16) KV_DECL_FUSED(0, 32)
KV_DECL_FUSED(1, 0) KV_DECL_FUSED(1, 2) KV_DECL_FUSED(1, 4) KV_DECL_FUSED(1, 8) KV_DECL_FUSED(1, 16) KV_DECL_FUSED(1, 32)
#undef KV_DECL_FUSED

// Picks the instantiation for sel (a W without a dedicated build uses the
// run-time-W kernel) and launches it over tiles [args.tile_lo, args.tile_hi).
hipError_t kv_launch_fused(const KvKernelSel& sel, const KvLaunchArgs& args, unsigned grid, hipStream_t stream);

// Plain float4 grid-stride copy of `bytes` bytes (multiple of 16).
hipError_t kv_launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);

// Copy preceded by `spin` dependent multiply-adds per lane (a compute-bound stand-in for a
// backward operator).
// The grid has at most max_blocks workgroups (0 = at most 2048).
hipError_t kv_launch_busy_copy(void* dst, const void* src, size_t bytes, int spin, int max_blocks, hipStream_t stream);

// Copies the keys whose tiles are [tile_lo, tile_hi) from an arena to dst_table[segment] (device
// table of one destination pointer per segment), one workgroup per tile.
hipError_t kv_launch_gather(const KvTile* tiles, int64_t tile_lo, int64_t tile_hi, const float* arena,
                            float* const* dst_table, hipStream_t stream);

// Reads `bytes` bytes (multiple of 16) and writes nothing: a measured ceiling for reads.
hipError_t kv_launch_read(const void* src, size_t bytes, hipStream_t stream);

// One pass over n_read (1, 2, 4, 8, 16 or 32) read buffers and n_write (0..8) written buffers of
// `bytes` bytes each (multiple of 16), read buffers first in `bufs` (host array of device pointers):
// every lane sums its 16-byte vector of the read buffers and stores the sum to every written buffer.
// A measured ceiling for a mix of streams.
hipError_t kv_launch_mix(void* const* bufs, int n_read, int n_write, size_t bytes, hipStream_t stream);

// Copies the current weights of the keys whose tiles are [tile_lo, tile_hi) to their replica buffers:
// rows is the device table [segments * n_rep] of replica pointers (a null first pointer: none for
// that key), replicas are fp32 or, with rep_f16, fp16 rounded to nearest even.
hipError_t kv_launch_replicate(const KvTile* tiles, int64_t tile_lo, int64_t tile_hi, const float* arena,
                               const void* const* rows, int n_rep, int rep_f16, hipStream_t stream);

// Allocation-free pointer table: one file-scope device array per GPU of KV_STATIC_TABLE_PTRS gradient
// pointers (512 KiB), filled by a kernel that carries up to KV_FILL_PTRS pointers per launch in its arguments.
constexpr int KV_STATIC_TABLE_PTRS = 65536;
constexpr int KV_FILL_PTRS = 384;
// Device address of that array on `device`, which must be the current device (looked up once per device).
hipError_t kv_static_table(int device, const void*** table_out);
// table[first + i] = host_ptrs[i] for i < n, on `stream`; no allocation and no host-to-device copy.
hipError_t kv_launch_fill_rows(const void** table, size_t first, const void* const* host_ptrs, size_t n, hipStream_t stream);

// Plain cached pass over `bytes` bytes (multiple of 16), loads only or (dirty) read-modify-write: leaves this
// buffer's lines, and nothing else, in the caches it is larger than.
hipError_t kv_launch_touch(void* buf, size_t bytes, bool dirty, hipStream_t stream);
// One empty workgroup.
hipError_t kv_launch_null(hipStream_t stream);
