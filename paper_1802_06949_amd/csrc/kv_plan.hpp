// Host-side bucket plan and launch-order chain (no GPU needed).
#pragma once
#include <stddef.h>
#include <stdint.h>

#include <vector>

#include "kv_device.hpp"

// Key starts in the w / m / s arenas are multiples of this many elements (256 bytes).
constexpr int64_t KV_ARENA_ALIGN_ELEMS = 64;

struct KvPlanUnit {
    std::vector<int> keys;   // ascending
    bool large = false;
    int seg_begin = 0;       // segments [seg_begin, seg_end) belong to this unit
    int seg_end = 0;
};

struct kv_plan {
    int num_keys = 0;
    int grad_dtype = 0;
    int itemsize = 4;
    size_t bucket_bytes = 0;
    std::vector<int64_t> numel;          // per key
    std::vector<int> key_unit;           // per key
    std::vector<int> key_seg;            // per key: segment index (launch order)
    std::vector<int64_t> key_arena_off;  // per key: element offset in the arenas
    std::vector<int> seg_key;            // per segment
    std::vector<KvPlanUnit> units;
    int64_t arena_numel = 0;
};

// Fills `plan`; returns a kv_status.
int kv_plan_build(kv_plan& plan, int num_keys, const int64_t* key_numel, int grad_dtype, size_t bucket_bytes);

// Cuts every key into tiles of tile_elems elements (the last one ragged), in
// (unit, key, offset) order.  unit_tile_begin gets num_units + 1 entries,
// seg_tile_begin num_segments + 1.
void kv_plan_tiles(const kv_plan& plan, int tile_elems, std::vector<KvTile>& tiles,
                   std::vector<int64_t>& unit_tile_begin, std::vector<int64_t>& seg_tile_begin);

struct kv_chain {
    const kv_plan* plan = nullptr;
    std::vector<int> pending;        // per unit: keys still missing for its next run
    std::vector<uint8_t> marked;     // per key
    int next_unit = 0;               // position in the launch order (0 = start of an iteration)
    int pending_keys = 0;            // marked keys whose unit has not run
    int launched_keys = 0;           // keys of the units that have run in the iteration in progress
    int64_t iteration = 0;
    bool descending = false;         // launch order runs from the last unit down to unit 0

    void reset(const kv_plan* p);
    int mark(int key);                          // kv_status
    // Next run of ready units: *first is its LOWEST unit index, *n its length.
    bool next_run(int* first, int* n);
};
