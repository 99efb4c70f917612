// Gradient-pointer table for callers that cannot allocate.
//
// The fused kernel finds the W gradient buffers of a key in a device table of
// [segments x W] pointers.  kv_push_list keeps such tables in memory from hipMalloc and fills
// them with copies from pinned staging memory.  kv_push_list_noalloc keeps its table in the
// file-scope array below, which the code object brings with it, and fills it with a small kernel
// whose pointers travel in the kernel arguments: no allocation, no host-to-device copy, and
// nothing a graph capture could not record.
//
// Every GPU the library runs on holds its own copy of the array, at its own address, until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// address a kernel can use is looked up once per device, below, and everything else works with
// that address.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "kv_kernels.hpp"

namespace {

static __device__ __align__(256) unsigned char scratch[KV_STATIC_TABLE_PTRS * sizeof(uint64_t)];

constexpr int MAX_DEVICES = 64;
std::mutex g_mu;
uint64_t* g_table[MAX_DEVICES] = {};           // device address of `scratch` on each device

struct FillArgs {
    uint64_t ptr[KV_FILL_PTRS];                 // travels by value in the kernel arguments
};

// table[first + i] = a.ptr[i], i < n.  One lane per pointer.
__global__ void __launch_bounds__(KV_THREADS) kv_fill_rows_kernel(uint64_t* __restrict__ table, uint32_t first, uint32_t n,
                                                                  const FillArgs a) {
    const uint32_t i = blockIdx.x * KV_THREADS + threadIdx.x;
    if (i < n) table[first + i] = a.ptr[i];
}

}  // namespace

hipError_t kv_static_table(int device, const void*** table_out) {
    if (device < 0 || device >= MAX_DEVICES || !table_out) return hipErrorInvalidValue;
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_table[device]) {
        int cur = -1;
        hipError_t e = hipGetDevice(&cur);
        if (e != hipSuccess) return e;
        if (cur != device) return hipErrorInvalidDevice;       // the lookup answers for the current device
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_table[device] = static_cast<uint64_t*>(p);
    }
    *table_out = reinterpret_cast<const void**>(g_table[device]);
    return hipSuccess;
}

hipError_t kv_launch_fill_rows(const void** table, size_t first, const void* const* host_ptrs, size_t n, hipStream_t stream) {
    if (!table || (n > 0 && !host_ptrs) || first + n > (size_t)KV_STATIC_TABLE_PTRS) return hipErrorInvalidValue;
    FillArgs a;
    for (size_t done = 0; done < n; done += KV_FILL_PTRS) {
        const size_t m = n - done < (size_t)KV_FILL_PTRS ? n - done : (size_t)KV_FILL_PTRS;
        for (size_t i = 0; i < m; ++i) a.ptr[i] = (uint64_t)(uintptr_t)host_ptrs[done + i];
        for (size_t i = m; i < (size_t)KV_FILL_PTRS; ++i) a.ptr[i] = 0;
        hipLaunchKernelGGL(kv_fill_rows_kernel, dim3((unsigned)((m + KV_THREADS - 1) / KV_THREADS)), dim3(KV_THREADS), 0, stream,
                           reinterpret_cast<uint64_t*>(table), (uint32_t)(first + done), (uint32_t)m, a);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}
