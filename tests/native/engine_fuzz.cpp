// Random programs through the dependency engine against sequential execution; built with
// ThreadSanitizer by tests/test_host_sanitizers.py.  CPU only: the GPU entry points the engine's
// ready-made operations call are stubbed.
#include <hip/hip_runtime_api.h>
#include "kv_engine.h"
#include <atomic>
#include <cstdio>
#include <vector>
#include <random>
extern "C" {
int kv_copy_bytes(void*, const void*, size_t, void*) { return 0; }
}
hipError_t kv_launch_busy_copy(void*, const void*, size_t, int, int, hipStream_t) { return hipSuccess; }
extern "C" {
int kv_push(kv_store*, int, const void* const*) { return 0; }
int kv_wait_event(kv_store*, void*) { return 0; }
}
struct Ctx { std::vector<long>* vals; int i; std::vector<int> r, w; };
static void run(void* a) { Ctx* c = (Ctx*)a; long acc = c->i + 1; for (int v : c->r) acc = (acc * 1000003 + (*c->vals)[v]) % 2147483647; for (int v : c->w) (*c->vals)[v] = ((*c->vals)[v] * 31 + acc) % 2147483647; }
int main() {
    for (int seed = 0; seed < 6; ++seed) {
        std::mt19937 g(seed); int V = 1 + g() % 8, N = 1000;
        std::vector<long> ref(V, 0), vals(V, 0); std::vector<Ctx> prog(N);
        for (int i = 0; i < N; ++i) { prog[i].i = i; int nr = g() % 4, nw = g() % 3; for (int k = 0; k < nr; ++k) prog[i].r.push_back(g() % V); for (int k = 0; k < nw; ++k) prog[i].w.push_back(g() % V); }
        for (auto& c : prog) { c.vals = &ref; Ctx d = c; /* engine dedups: reads that are also writes count as writes */ run(&d); }
        kv_engine* e; kv_engine_create(&e, 8); std::vector<int> tags(V); for (int& t : tags) kv_engine_new_var(e, &t);
        for (auto& c : prog) { c.vals = &vals; std::vector<int> r, w; for (int v : c.r) r.push_back(tags[v]); for (int v : c.w) w.push_back(tags[v]); kv_engine_push(e, run, &c, r.data(), (int)r.size(), w.data(), (int)w.size()); }
        kv_engine_wait_all(e); kv_engine_destroy(e);
        if (ref != vals) { printf("MISMATCH seed %d\n", seed); return 1; }
    }
    printf("tsan engine ok\n"); return 0;
}
