// A stand-in for the HIP runtime and for the library's kernel launchers, for CPU-only tests of the store's
// host logic (tests/native/alloc_count.cpp).  "Device" memory is host memory, copies are memcpy, kernels do
// nothing, streams run nothing asynchronously.  Every allocating runtime call is counted.
#include <hip/hip_runtime_api.h>

#include <cstdlib>
#include <cstring>

#include "kv_kernels.hpp"

long g_stub_device_allocs = 0;     // hipMalloc + hipHostMalloc
long g_stub_launches = 0;          // fused launches
long g_stub_fills = 0;             // row fills of the static table

namespace {
struct FakeEvent { int recorded; };
void* g_static[KV_STATIC_TABLE_PTRS];
}

extern "C" {
hipError_t hipGetDevice(int* d) { *d = 0; return hipSuccess; }
hipError_t hipDeviceGetAttribute(int* v, hipDeviceAttribute_t, int) { *v = 256; return hipSuccess; }
hipError_t hipMalloc(void** p, size_t n) { ++g_stub_device_allocs; *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipFree(void* p) { std::free(p); return hipSuccess; }
hipError_t hipHostMalloc(void** p, size_t n, unsigned) { ++g_stub_device_allocs; *p = std::malloc(n ? n : 1); return *p ? hipSuccess : hipErrorOutOfMemory; }
hipError_t hipHostFree(void* p) { std::free(p); return hipSuccess; }
hipError_t hipMemcpy(void* d, const void* s, size_t n, hipMemcpyKind) { std::memcpy(d, s, n); return hipSuccess; }
hipError_t hipMemcpyAsync(void* d, const void* s, size_t n, hipMemcpyKind, hipStream_t) { std::memmove(d, s, n); return hipSuccess; }
hipError_t hipMemset(void* d, int v, size_t n) { std::memset(d, v, n); return hipSuccess; }
hipError_t hipMemsetAsync(void* d, int v, size_t n, hipStream_t) { std::memset(d, v, n); return hipSuccess; }
hipError_t hipEventCreate(hipEvent_t* e) { *e = reinterpret_cast<hipEvent_t>(new FakeEvent{0}); return hipSuccess; }
hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) { return hipEventCreate(e); }
hipError_t hipEventDestroy(hipEvent_t e) { delete reinterpret_cast<FakeEvent*>(e); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t e, hipStream_t) { reinterpret_cast<FakeEvent*>(e)->recorded++; return hipSuccess; }
hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 1.0f; return hipSuccess; }
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned) { *s = reinterpret_cast<hipStream_t>(new int(0)); return hipSuccess; }
hipError_t hipStreamDestroy(hipStream_t s) { delete reinterpret_cast<int*>(s); return hipSuccess; }
hipError_t hipStreamIsCapturing(hipStream_t, hipStreamCaptureStatus* st) { *st = hipStreamCaptureStatusNone; return hipSuccess; }
hipError_t hipGetLastError(void) { return hipSuccess; }
const char* hipGetErrorString(hipError_t) { return "stub"; }
}

hipError_t kv_launch_fused(const KvKernelSel&, const KvLaunchArgs&, unsigned, hipStream_t) { ++g_stub_launches; return hipSuccess; }
hipError_t kv_launch_gather(const KvTile*, int64_t, int64_t, const float*, float* const*, hipStream_t) { return hipSuccess; }
hipError_t kv_launch_replicate(const KvTile*, int64_t, int64_t, const float*, const void* const*, int, int, hipStream_t) { return hipSuccess; }
hipError_t kv_static_table(int, const void*** out) { *out = const_cast<const void**>(reinterpret_cast<void**>(g_static)); return hipSuccess; }
hipError_t kv_launch_fill_rows(const void** table, size_t first, const void* const* ptrs, size_t n, hipStream_t) {
    ++g_stub_fills;
    if (first + n > (size_t)KV_STATIC_TABLE_PTRS) return hipErrorInvalidValue;
    for (size_t i = 0; i < n; ++i) table[first + i] = ptrs[i];
    return hipSuccess;
}
