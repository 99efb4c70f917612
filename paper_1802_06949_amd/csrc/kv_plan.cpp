// Bucket packing, arena layout, tiling and the in-order launch chain.
//
// The paper keeps one communication buffer per key and orders its collectives by
// chaining them on a dummy write dependency ("MPI Dependency Chaining").  Here the
// order is fixed once, from the key set alone: keys are packed into units and the
// units run in ascending index.
#include "kv_plan.hpp"

#include "../../include/kv.h"

int kv_plan_build(kv_plan& plan, int num_keys, const int64_t* key_numel, int grad_dtype, size_t bucket_bytes) {
    if (num_keys < 1 || !key_numel || bucket_bytes < 1) return KV_ERR_ARG;
    if (grad_dtype != KV_F32 && grad_dtype != KV_F16) return KV_ERR_ARG;
    for (int k = 0; k < num_keys; ++k)
        if (key_numel[k] < 0) return KV_ERR_ARG;

    plan = kv_plan();
    plan.num_keys = num_keys;
    plan.grad_dtype = grad_dtype;
    plan.itemsize = grad_dtype == KV_F16 ? 2 : 4;
    plan.bucket_bytes = bucket_bytes;
    plan.numel.assign(key_numel, key_numel + num_keys);
    plan.key_unit.assign(num_keys, -1);

    // Pass 1: units in order of their first key.  The open bucket survives large keys.
    int open = -1;                 // index into plan.units of the bucket still accepting keys
    unsigned __int128 open_bytes = 0;
    for (int k = 0; k < num_keys; ++k) {
        const unsigned __int128 size = (unsigned __int128)key_numel[k] * (unsigned)plan.itemsize;
        if (size >= bucket_bytes) {
            KvPlanUnit u;
            u.large = true;
            u.keys.push_back(k);
            plan.key_unit[k] = (int)plan.units.size();
            plan.units.push_back(u);
            continue;
        }
        if (open >= 0 && open_bytes + size <= bucket_bytes) {
            plan.units[open].keys.push_back(k);
            open_bytes += size;
        } else {
            KvPlanUnit u;
            u.keys.push_back(k);
            open = (int)plan.units.size();
            open_bytes = size;
            plan.units.push_back(u);
        }
        plan.key_unit[k] = open;
    }

    // Pass 2: segments and arena offsets, units in index order, keys ascending.
    plan.key_seg.assign(num_keys, -1);
    plan.key_arena_off.assign(num_keys, 0);
    int64_t cur = 0;
    for (auto& u : plan.units) {
        u.seg_begin = (int)plan.seg_key.size();
        for (int k : u.keys) {
            // Every key starts on a 256-byte boundary of the arenas, so that a wavefront's accesses to w and m cover
            // whole 128-byte lines whatever the sizes of the keys before it.  (With 16-byte alignment one key of
            // 1000 elements put every later key 32 bytes off the line grid, and write-through stores of part of
            // a line are slow: one key of 25.6 M elements behind a 4-element key ran in 201 us instead of 161 us.)
            cur = (cur + (KV_ARENA_ALIGN_ELEMS - 1)) & ~(int64_t)(KV_ARENA_ALIGN_ELEMS - 1);
            plan.key_arena_off[k] = cur;
            plan.key_seg[k] = (int)plan.seg_key.size();
            plan.seg_key.push_back(k);
            cur += plan.numel[k];
        }
        u.seg_end = (int)plan.seg_key.size();
    }
    plan.arena_numel = (cur + (KV_ARENA_ALIGN_ELEMS - 1)) & ~(int64_t)(KV_ARENA_ALIGN_ELEMS - 1);
    return KV_OK;
}

void kv_plan_tiles(const kv_plan& plan, int tile_elems, std::vector<KvTile>& tiles,
                   std::vector<int64_t>& unit_tile_begin, std::vector<int64_t>& seg_tile_begin) {
    tiles.clear();
    unit_tile_begin.clear();
    seg_tile_begin.clear();
    for (const auto& u : plan.units) {
        unit_tile_begin.push_back((int64_t)tiles.size());
        for (int k : u.keys) {
            seg_tile_begin.push_back((int64_t)tiles.size());         // segments are numbered in this order
            for (int64_t off = 0; off < plan.numel[k]; off += tile_elems) {
                KvTile t;
                t.seg = plan.key_seg[k];
                const int64_t left = plan.numel[k] - off;
                t.count = (int32_t)(left < tile_elems ? left : tile_elems);
                t.arena_off = plan.key_arena_off[k] + off;
                t.seg_off = off;
                t.reserved = 0;
                tiles.push_back(t);
            }
        }
    }
    unit_tile_begin.push_back((int64_t)tiles.size());
    seg_tile_begin.push_back((int64_t)tiles.size());
}

void kv_chain::reset(const kv_plan* p) {
    plan = p;
    pending.clear();
    for (const auto& u : p->units) pending.push_back((int)u.keys.size());
    marked.assign(p->num_keys, 0);
    next_unit = 0;
    pending_keys = 0;
    launched_keys = 0;
    iteration = 0;
}

int kv_chain::mark(int key) {
    if (key < 0 || key >= plan->num_keys) return KV_ERR_KEY;
    if (marked[key]) return KV_ERR_STATE;
    marked[key] = 1;
    --pending[plan->key_unit[key]];
    ++pending_keys;
    return KV_OK;
}

bool kv_chain::next_run(int* first, int* n) {
    const int U = (int)plan->units.size();
    auto unit_at = [&](int pos) { return descending ? U - 1 - pos : pos; };
    if (pending[unit_at(next_unit)] != 0) return false;
    const int pos0 = next_unit;
    while (next_unit < U && pending[unit_at(next_unit)] == 0) {
        const int ui = unit_at(next_unit);
        const auto& u = plan->units[ui];
        pending[ui] = (int)u.keys.size();
        for (int k : u.keys) marked[k] = 0;
        pending_keys -= (int)u.keys.size();
        launched_keys += (int)u.keys.size();
        ++next_unit;
    }
    *n = next_unit - pos0;
    *first = descending ? U - next_unit : pos0;      // lowest unit of the run
    if (next_unit == U) {
        next_unit = 0;
        launched_keys = 0;
        ++iteration;
    }
    return true;
}
