// Kernel selection and the plain copy kernel.
#include <hip/hip_runtime.h>

#include "kv_kernels.hpp"

hipError_t kv_launch_fused(const KvKernelSel& sel, const KvLaunchArgs& args, unsigned grid, hipStream_t stream) {
    if (args.tile_hi <= args.tile_lo || grid == 0) return hipSuccess;
#define KV_CASE(W) \
    case W: return sel.grad_f16 ? kv_launch_fused_f1_w##W(sel, args, grid, stream) \
                                : kv_launch_fused_f0_w##W(sel, args, grid, stream);
    switch (sel.generic_w ? 0 : sel.W) {
        KV_CASE(2) KV_CASE(4) KV_CASE(8) KV_CASE(16) KV_CASE(32)
        default: break;
    }
#undef KV_CASE
    return sel.grad_f16 ? kv_launch_fused_f1_w0(sel, args, grid, stream) : kv_launch_fused_f0_w0(sel, args, grid, stream);
}

namespace {
typedef float f32x4 __attribute__((ext_vector_type(4)));

__global__ void __launch_bounds__(KV_THREADS) kv_copy_kernel(f32x4* __restrict__ dst, const f32x4* __restrict__ src, size_t nvec) {
    const size_t stride = (size_t)gridDim.x * KV_THREADS;
    for (size_t i = (size_t)blockIdx.x * KV_THREADS + threadIdx.x; i < nvec; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}
// Reads `nvec` 16-byte vectors with the non-temporal hint and writes nothing: the sum can never
// equal the sentinel, but the compiler cannot know that.
__global__ void __launch_bounds__(KV_THREADS) kv_read_kernel(const f32x4* __restrict__ src, size_t nvec, f32x4* sink) {
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    const size_t stride = (size_t)gridDim.x * KV_THREADS;
    for (size_t i = (size_t)blockIdx.x * KV_THREADS + threadIdx.x; i < nvec; i += stride)
        acc += __builtin_nontemporal_load(src + i);
    if (acc.x == -12345.678f && acc.y == 3.25f) sink[0] = acc;
}

// Plain cached loads and stores: every line of the buffer passes through L2 and the memory-side cache.
template <bool DIRTY>
__global__ void __launch_bounds__(KV_THREADS) kv_touch_kernel(f32x4* __restrict__ buf, size_t nvec) {
    const size_t stride = (size_t)gridDim.x * KV_THREADS;
    f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (size_t i = (size_t)blockIdx.x * KV_THREADS + threadIdx.x; i < nvec; i += stride) {
        f32x4 v = buf[i];
        if constexpr (DIRTY) {
            v.x += 1.0f;
            buf[i] = v;
        } else {
            acc += v;
        }
    }
    // the sum can never equal the sentinel, but the compiler cannot know that, so the loads stay
    if (!DIRTY && acc.x == -12345.678f && acc.y == 3.25f) buf[0] = acc;
}
__global__ void kv_null_kernel() {}

// R read streams and n_write written streams with the access pattern of the fused kernel: one
// workgroup per 4 KB tile of every stream, every load in flight before the first store.
struct KvMixArgs {
    const f32x4* rd[32];
    f32x4* wr[8];
};
template <int R>
__global__ void __launch_bounds__(KV_THREADS) kv_mix_kernel(const KvMixArgs a, int n_write, size_t nvec) {
    const size_t i = (size_t)blockIdx.x * KV_THREADS + threadIdx.x;
    if (i >= nvec) return;
    f32x4 v[R];
#pragma unroll
    for (int s = 0; s < R; ++s) v[s] = __builtin_nontemporal_load(a.rd[s] + i);
    f32x4 acc = v[0];
#pragma unroll
    for (int s = 1; s < R; ++s) acc += v[s];
    for (int s = 0; s < n_write; ++s) a.wr[s][i] = acc;
    // with no written stream the sum goes nowhere; it can never equal the sentinel, but the compiler cannot know
    if (n_write == 0 && acc.x == -12345.678f && acc.y == 3.25f) const_cast<f32x4*>(a.rd[0])[i] = acc;
}

// Stand-in for a compute-bound backward operator: every lane first runs `spin` dependent
// multiply-adds (no memory traffic), then copies its share.  The spun value can never equal
// the sentinel, but the compiler cannot know that, so the loop stays.
__global__ void __launch_bounds__(KV_THREADS) kv_busy_copy_kernel(f32x4* __restrict__ dst, const f32x4* __restrict__ src,
                                                                  size_t nvec, int spin) {
    float x = 1.0f + 1e-7f * (float)threadIdx.x;
    for (int i = 0; i < spin; ++i) x = x * 0.9999999f + 1e-9f;
    const size_t stride = (size_t)gridDim.x * KV_THREADS;
    for (size_t i = (size_t)blockIdx.x * KV_THREADS + threadIdx.x; i < nvec; i += stride) {
        f32x4 v = src[i];
        if (x == -12345.0f) v.x = x;
        dst[i] = v;
    }
}
// Gather of whole keys out of an arena: tile t of the store's tile table is copied to
// dst[segment of t] + its offset inside the key.  One wavefront per tile (a tile may be as small
// as 256 elements, one 16-byte vector per lane), four tiles per workgroup.  The copies are an output
// stream: non-temporal stores keep them from pushing w and m out of the memory-side cache.
__global__ void __launch_bounds__(KV_THREADS) kv_gather_kernel(const KvTile* __restrict__ tiles, int64_t tile_lo,
                                                               int64_t tile_hi, const float* __restrict__ arena,
                                                               float* const* __restrict__ dst) {
    constexpr int WAVES = KV_THREADS / 64;
    const int64_t t = tile_lo + (int64_t)blockIdx.x * WAVES + (threadIdx.x >> 6);
    if (t >= tile_hi) return;
    const KvTile td = tiles[t];
    const float* __restrict__ src = arena + td.arena_off;
    float* __restrict__ out = dst[td.seg] + td.seg_off;
    const int lane = threadIdx.x & 63;
    if ((reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
        const int nvec = td.count >> 2;
        for (int v = lane; v < nvec; v += 64)
            __builtin_nontemporal_store(reinterpret_cast<const f32x4*>(src)[v], reinterpret_cast<f32x4*>(out) + v);
        const int k = (nvec << 2) + lane;
        if (k < td.count) __builtin_nontemporal_store(src[k], out + k);
    } else {
        for (int k = lane; k < td.count; k += 64) __builtin_nontemporal_store(src[k], out + k);
    }
}
// Copies the current weights of the keys whose tiles are [tile_lo, tile_hi) to their replica buffers
// (rows of n_rep pointers per segment; a null first pointer: the key has no replicas), as fp32 or rounded
// to nearest-even fp16.  One wavefront per tile, non-temporal stores (the replicas are output streams).
__global__ void __launch_bounds__(KV_THREADS) kv_replicate_kernel(const KvTile* __restrict__ tiles, int64_t tile_lo,
                                                                  int64_t tile_hi, const float* __restrict__ arena,
                                                                  const void* const* __restrict__ rows, int n_rep,
                                                                  int rep_f16) {
    typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
    constexpr int WAVES = KV_THREADS / 64;
    const int64_t t = tile_lo + (int64_t)blockIdx.x * WAVES + (threadIdx.x >> 6);
    if (t >= tile_hi) return;
    const KvTile td = tiles[t];
    const void* const* row = rows + (int64_t)td.seg * n_rep;
    if (row[0] == nullptr) return;
    const float* __restrict__ src = arena + td.arena_off;
    const int lane = threadIdx.x & 63;
    uintptr_t bits = 0;
    for (int r = 0; r < n_rep; ++r) bits |= reinterpret_cast<uintptr_t>(row[r]);
    const bool vec_ok = (bits & (rep_f16 ? 7u : 15u)) == 0;      // seg_off is a multiple of 4 elements
    const int nvec = vec_ok ? td.count >> 2 : 0;
    for (int v = lane; v < nvec; v += 64) {
        const f32x4 x = reinterpret_cast<const f32x4*>(src)[v];
        if (rep_f16) {
            f16x4 h;
            for (int c = 0; c < 4; ++c) h[c] = (_Float16)x[c];
            for (int r = 0; r < n_rep; ++r)
                __builtin_nontemporal_store(h, reinterpret_cast<f16x4*>((_Float16*)row[r] + td.seg_off) + v);
        } else {
            for (int r = 0; r < n_rep; ++r)
                __builtin_nontemporal_store(x, reinterpret_cast<f32x4*>((float*)row[r] + td.seg_off) + v);
        }
    }
    for (int k = (nvec << 2) + lane; k < td.count; k += 64) {
        const float x = src[k];
        for (int r = 0; r < n_rep; ++r) {
            if (rep_f16) __builtin_nontemporal_store((_Float16)x, (_Float16*)row[r] + td.seg_off + k);
            else __builtin_nontemporal_store(x, (float*)row[r] + td.seg_off + k);
        }
    }
}
}  // namespace

hipError_t kv_launch_replicate(const KvTile* tiles, int64_t tile_lo, int64_t tile_hi, const float* arena,
                               const void* const* rows, int n_rep, int rep_f16, hipStream_t stream) {
    if (tile_hi <= tile_lo || n_rep <= 0) return hipSuccess;
    constexpr int64_t waves = KV_THREADS / 64;
    hipLaunchKernelGGL(kv_replicate_kernel, dim3((unsigned)((tile_hi - tile_lo + waves - 1) / waves)), dim3(KV_THREADS), 0,
                       stream, tiles, tile_lo, tile_hi, arena, rows, n_rep, rep_f16);
    return hipGetLastError();
}

hipError_t kv_launch_gather(const KvTile* tiles, int64_t tile_lo, int64_t tile_hi, const float* arena,
                            float* const* dst_table, hipStream_t stream) {
    if (tile_hi <= tile_lo) return hipSuccess;
    constexpr int64_t waves = KV_THREADS / 64;
    hipLaunchKernelGGL(kv_gather_kernel, dim3((unsigned)((tile_hi - tile_lo + waves - 1) / waves)), dim3(KV_THREADS), 0,
                       stream, tiles, tile_lo, tile_hi, arena, dst_table);
    return hipGetLastError();
}

hipError_t kv_launch_read(const void* src, size_t bytes, hipStream_t stream) {
    const size_t nvec = bytes / 16;
    if (nvec == 0) return hipSuccess;
    size_t blocks = (nvec + KV_THREADS - 1) / KV_THREADS;
    if (blocks > (1u << 22)) blocks = 1u << 22;
    hipLaunchKernelGGL(kv_read_kernel, dim3((unsigned)blocks), dim3(KV_THREADS), 0, stream,
                       static_cast<const f32x4*>(src), nvec, const_cast<f32x4*>(static_cast<const f32x4*>(src)));
    return hipGetLastError();
}

hipError_t kv_launch_busy_copy(void* dst, const void* src, size_t bytes, int spin, int max_blocks, hipStream_t stream) {
    const size_t nvec = bytes / 16;
    if (nvec == 0) return hipSuccess;
    size_t blocks = (nvec + KV_THREADS - 1) / KV_THREADS;
    const size_t cap = max_blocks > 0 && max_blocks < 256 * 8 ? (size_t)max_blocks : 256u * 8u;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(kv_busy_copy_kernel, dim3((unsigned)blocks), dim3(KV_THREADS), 0, stream,
                       static_cast<f32x4*>(dst), static_cast<const f32x4*>(src), nvec, spin);
    return hipGetLastError();
}

hipError_t kv_launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream) {
    const size_t nvec = bytes / 16;
    if (nvec == 0) return hipSuccess;
    size_t blocks = (nvec + KV_THREADS - 1) / KV_THREADS;      // one vector per lane: the fastest shape measured
    if (blocks > (1u << 22)) blocks = 1u << 22;
    hipLaunchKernelGGL(kv_copy_kernel, dim3((unsigned)blocks), dim3(KV_THREADS), 0, stream,
                       static_cast<f32x4*>(dst), static_cast<const f32x4*>(src), nvec);
    return hipGetLastError();
}

hipError_t kv_launch_mix(void* const* bufs, int n_read, int n_write, size_t bytes, hipStream_t stream) {
    const size_t nvec = bytes / 16;
    if (nvec == 0) return hipSuccess;
    const size_t blocks = (nvec + KV_THREADS - 1) / KV_THREADS;
    if (n_read > 32 || n_write > 8 || blocks > 0x7FFFFFFFu) return hipErrorInvalidValue;
    KvMixArgs a{};
    for (int s = 0; s < n_read; ++s) a.rd[s] = static_cast<const f32x4*>(bufs[s]);
    for (int s = 0; s < n_write; ++s) a.wr[s] = static_cast<f32x4*>(bufs[n_read + s]);
#define KV_MIX(R) \
    case R: hipLaunchKernelGGL(kv_mix_kernel<R>, dim3((unsigned)blocks), dim3(KV_THREADS), 0, stream, a, n_write, nvec); break;
    switch (n_read) {
        KV_MIX(1) KV_MIX(2) KV_MIX(4) KV_MIX(8) KV_MIX(16) KV_MIX(32)
        default: return hipErrorInvalidValue;
    }
#undef KV_MIX
    return hipGetLastError();
}

hipError_t kv_launch_touch(void* buf, size_t bytes, bool dirty, hipStream_t stream) {
    const size_t nvec = bytes / 16;
    if (nvec == 0) return hipSuccess;
    size_t blocks = (nvec + KV_THREADS - 1) / KV_THREADS;
    if (blocks > (1u << 22)) blocks = 1u << 22;
    if (dirty) hipLaunchKernelGGL(kv_touch_kernel<true>, dim3((unsigned)blocks), dim3(KV_THREADS), 0, stream, static_cast<f32x4*>(buf), nvec);
    else hipLaunchKernelGGL(kv_touch_kernel<false>, dim3((unsigned)blocks), dim3(KV_THREADS), 0, stream, static_cast<f32x4*>(buf), nvec);
    return hipGetLastError();
}

hipError_t kv_launch_null(hipStream_t stream) {
    hipLaunchKernelGGL(kv_null_kernel, dim3(1), dim3(64), 0, stream);
    return hipGetLastError();
}
