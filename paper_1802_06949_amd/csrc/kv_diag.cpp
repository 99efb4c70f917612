// Measurement helpers declared in include/kv_diag.h: plain kernels of known size, measured ceilings,
// a cache flush and an empty launch.  Not part of the method.
#include <hip/hip_runtime_api.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>

#include "../../include/kv.h"
#include "../../include/kv_diag.h"
#include "kv_error.hpp"
#include "kv_kernels.hpp"

namespace {
void fail(const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    kv_set_global_error(buf);
}
}  // namespace

extern "C" {

int kv_copy_bytes(void* dev_dst, const void* dev_src, size_t bytes, void* hip_stream) {
    if (!dev_dst || !dev_src || (bytes & 15u) || ((uintptr_t)dev_dst & 15u) || ((uintptr_t)dev_src & 15u)) {
        fail("kv_copy_bytes: pointers and size must be multiples of 16");
        return KV_ERR_ARG;
    }
    hipError_t e = kv_launch_copy(dev_dst, dev_src, bytes, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) {
        fail("kv_copy_bytes: %s", hipGetErrorString(e));
        return KV_ERR_HIP;
    }
    return KV_OK;
}

int kv_read_bytes(const void* dev_src, size_t bytes, void* hip_stream) {
    if (!dev_src || (bytes & 15u) || ((uintptr_t)dev_src & 15u)) {
        fail("kv_read_bytes: pointer and size must be multiples of 16");
        return KV_ERR_ARG;
    }
    hipError_t e = kv_launch_read(dev_src, bytes, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) {
        fail("kv_read_bytes: %s", hipGetErrorString(e));
        return KV_ERR_HIP;
    }
    return KV_OK;
}

int kv_stream_mix(void* const* dev_bufs, int n_read, int n_write, size_t bytes, void* hip_stream) {
    const bool r_ok = n_read == 1 || n_read == 2 || n_read == 4 || n_read == 8 || n_read == 16 || n_read == 32;
    if (!dev_bufs || !r_ok || n_write < 0 || n_write > 8 || (bytes & 15u)) {
        fail("kv_stream_mix: n_read must be 1, 2, 4, 8, 16 or 32, n_write 0..8, bytes a multiple of 16");
        return KV_ERR_ARG;
    }
    for (int s = 0; s < n_read + n_write; ++s) {
        if (!dev_bufs[s] || ((uintptr_t)dev_bufs[s] & 15u)) {
            fail("kv_stream_mix: buffer %d is null or not aligned to 16 bytes", s);
            return KV_ERR_ARG;
        }
    }
    hipError_t e = kv_launch_mix(dev_bufs, n_read, n_write, bytes, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) {
        fail("kv_stream_mix: %s", hipGetErrorString(e));
        return KV_ERR_HIP;
    }
    return KV_OK;
}

int kv_evict_caches(void* dev_buf, size_t bytes, int dirty, void* hip_stream) {
    if (!dev_buf || (bytes & 15u) || ((uintptr_t)dev_buf & 15u)) {
        fail("kv_evict_caches: pointer and size must be multiples of 16");
        return KV_ERR_ARG;
    }
    hipError_t e = kv_launch_touch(dev_buf, bytes, dirty != 0, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) {
        fail("kv_evict_caches: %s", hipGetErrorString(e));
        return KV_ERR_HIP;
    }
    return KV_OK;
}

int kv_null_launch(int count, void* hip_stream) {
    if (count < 1) {
        fail("kv_null_launch: count must be at least 1");
        return KV_ERR_ARG;
    }
    hipError_t e = hipSuccess;
    for (int i = 0; i < count && e == hipSuccess; ++i) e = kv_launch_null(static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) {
        fail("kv_null_launch: %s", hipGetErrorString(e));
        return KV_ERR_HIP;
    }
    return KV_OK;
}

int kv_push_list_repeat(kv_store* store, int nkeys, const int* keys, const void* const* dev_grads, int reps) {
    if (reps < 1) {
        fail("kv_push_list_repeat: reps must be at least 1");
        return KV_ERR_ARG;
    }
    for (int i = 0; i < reps; ++i) {
        const int rc = kv_push_list(store, nkeys, keys, dev_grads);
        if (rc != KV_OK) return rc;
    }
    return KV_OK;
}

}  // extern "C"
