// The store's steady state allocates nothing: whole iterations of push / pull / wait / barrier are run against a
// stand-in HIP runtime (hip_stub.cpp) while every operator new and every allocating runtime call is counted.
// Built and run by tests/test_host_sanitizers.py.  CPU only.
#include <cstdio>
#include <cstdlib>
#include <new>
#include <vector>

#include "kv.h"

static long g_news = 0;
void* operator new(std::size_t n) { ++g_news; void* p = std::malloc(n ? n : 1); if (!p) throw std::bad_alloc(); return p; }
void* operator new[](std::size_t n) { ++g_news; void* p = std::malloc(n ? n : 1); if (!p) throw std::bad_alloc(); return p; }
void* operator new(std::size_t n, const std::nothrow_t&) noexcept { ++g_news; return std::malloc(n ? n : 1); }
void operator delete(void* p) noexcept { std::free(p); }
void operator delete[](void* p) noexcept { std::free(p); }
void operator delete(void* p, std::size_t) noexcept { std::free(p); }
void operator delete[](void* p, std::size_t) noexcept { std::free(p); }

extern long g_stub_device_allocs, g_stub_launches, g_stub_fills;

#define REQUIRE(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

struct Counts { long news, dev; };
static Counts now() { return Counts{g_news, g_stub_device_allocs}; }

int main() {
    const int K = 40, W = 4;
    std::vector<int64_t> numel(K);
    for (int k = 0; k < K; ++k) numel[k] = k % 7 == 0 ? 300000 : 100 + 37 * k;
    kv_sgd_params p{0.1f, 0.9f, 1e-4f, 0.0f, KV_REDUCE_SEQUENTIAL};
    // "device" buffers: any distinct, aligned addresses do, the stub never reads them
    std::vector<std::vector<float>> grads(2 * K * W, std::vector<float>(4));
    std::vector<const void*> ptrs[2];
    for (int s = 0; s < 2; ++s)
        for (int i = 0; i < K * W; ++i) ptrs[s].push_back(grads[(size_t)s * K * W + i].data());
    std::vector<int> keys(K);
    for (int k = 0; k < K; ++k) keys[k] = k;
    std::vector<float> out(300000);
    std::vector<void*> outs(K, out.data());

    for (unsigned flags : {0u, (unsigned)KV_FLAG_LAZY_LAUNCH, (unsigned)KV_FLAG_KEEP_SUM}) {
        kv_store* st = nullptr;
        const Counts at_start = now();
        REQUIRE(kv_init(&st, K, numel.data(), KV_F32, W, 64 << 10, &p, flags, nullptr, nullptr) == KV_OK);
        REQUIRE(g_news > at_start.news && g_stub_device_allocs > at_start.dev);        // the counters do see kv_init
        auto iteration = [&](int s, int mode) -> int {
            if (mode == 0) {                                    // one list push
                REQUIRE(kv_push_list(st, K, keys.data(), ptrs[s].data()) == KV_OK);
            } else if (mode == 1) {                             // single pushes, last key first, pulls queued in between
                for (int k = K - 1; k >= 0; --k) {
                    REQUIRE(kv_push(st, k, ptrs[s].data() + (size_t)k * W) == KV_OK);
                    if (k % 5 == 0) REQUIRE(kv_pull(st, k, out.data()) == KV_OK);
                    if (k % 9 == 0) REQUIRE(kv_pull_momentum(st, k, out.data()) == KV_OK);
                }
            } else {                                            // the allocation-free list push
                REQUIRE(kv_push_list_noalloc(st, K, keys.data(), ptrs[s].data()) == KV_OK);
            }
            REQUIRE(kv_pull(st, 3, out.data()) == KV_OK);
            REQUIRE(kv_pull_list(st, K, keys.data(), outs.data()) == KV_OK);
            REQUIRE(kv_wait(st, 7) == KV_OK);
            REQUIRE(kv_barrier(st) == KV_OK);
            REQUIRE(kv_wait(st, -1) == KV_OK);
            return 0;
        };
        // warm-up: both gradient sets reach the cached tables, every path has run once
        for (int mode = 0; mode < 3; ++mode)
            for (int s = 0; s < 2; ++s)
                if (iteration(s, mode)) return 1;
        const Counts before = now();
        const long launches_before = g_stub_launches;
        for (int rep = 0; rep < 20; ++rep)
            for (int mode = 0; mode < 3; ++mode)
                if (iteration(rep & 1, mode)) return 1;
        const Counts after = now();
        REQUIRE(g_stub_launches > launches_before);
        if (after.news != before.news || after.dev != before.dev) {
            std::printf("FAILED: flags %u: %ld host allocations and %ld device allocations in steady state\n", flags,
                        after.news - before.news, after.dev - before.dev);
            return 1;
        }
        // the other schedules, after their own warm-up
        for (int sched : {KV_SCHED_FUNNEL, KV_SCHED_CONCURRENT}) {
            REQUIRE(kv_set_schedule(st, sched, 4, 8) == KV_OK);
            if (iteration(0, 0) || iteration(1, 1)) return 1;
            const Counts b2 = now();
            for (int rep = 0; rep < 6; ++rep)
                if (iteration(rep & 1, rep % 2)) return 1;
            const Counts a2 = now();
            if (a2.news != b2.news || a2.dev != b2.dev) {
                std::printf("FAILED: schedule %d: %ld host / %ld device allocations in steady state\n", sched, a2.news - b2.news,
                            a2.dev - b2.dev);
                return 1;
            }
        }
        REQUIRE(kv_set_schedule(st, KV_SCHED_CHAINED, 1, 0) == KV_OK);
        kv_destroy(st);
    }
    REQUIRE(g_stub_fills > 0);
    std::printf("steady state allocates nothing: ok\n");
    return 0;
}
