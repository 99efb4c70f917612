// Random key sets through the bucket plan, the tiling and the launch chain; built with
// AddressSanitizer + UBSan by tests/test_host_sanitizers.py.  CPU only.
#include "kv_plan.hpp"
#include "kv.h"
#include <cstdio>
#include <random>
#include <algorithm>
int main() {
    std::mt19937_64 g(1);
    for (int it = 0; it < 400; ++it) {
        int K = 1 + g() % 80; std::vector<int64_t> n(K);
        for (auto& x : n) { int c = g() % 6; x = c == 0 ? 0 : c == 1 ? g() % 10 : c == 2 ? g() % 5000 : c == 3 ? 4096 : c == 4 ? g() % 3000000 : (int64_t)1 << (g() % 33); }
        size_t bucket = (size_t)1 << (g() % 40); if (g() % 5 == 0) bucket += g() % 100;
        kv_plan p; int dt = g() % 2;
        if (kv_plan_build(p, K, n.data(), dt, bucket) != KV_OK) { printf("build failed\n"); return 1; }
        std::vector<KvTile> tiles; std::vector<int64_t> ub, sb;
        int te = kv_tile_elems(1 << (g() % 3), 1 << (g() % 3));
        int64_t total_tiles = 0; for (auto x : n) total_tiles += (x + te - 1) / te;
        if (total_tiles < 300000) { kv_plan_tiles(p, te, tiles, ub, sb); if ((int64_t)tiles.size() != total_tiles) { printf("tiles\n"); return 1; } }
        kv_chain c; c.reset(&p); c.descending = g() % 2;
        std::vector<int> perm(K); for (int i = 0; i < K; ++i) perm[i] = i;
        for (int rep = 0; rep < 2; ++rep) {
            std::shuffle(perm.begin(), perm.end(), g); int launched = 0;
            for (int k : perm) { if (c.mark(k) != KV_OK) { printf("mark\n"); return 1; } int f, m; while (c.next_run(&f, &m)) launched += m; }
            if (launched != (int)p.units.size() || c.pending_keys != 0 || c.next_unit != 0) { printf("chain\n"); return 1; }
        }
        if (c.mark(-1) != KV_ERR_KEY || c.mark(K) != KV_ERR_KEY) return 1;
    }
    printf("asan/ubsan plan+chain ok\n"); return 0;
}
