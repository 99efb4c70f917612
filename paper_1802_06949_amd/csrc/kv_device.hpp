// Structures shared by the host scheduler and the kernels.
#pragma once
#include <stdint.h>

constexpr int KV_THREADS = 256;          // 4 wavefronts of 64 lanes per workgroup

// One tile: a contiguous piece of one key handled by one workgroup pass.
// Element counts; seg_off is a multiple of the tile size, so 16-byte vectors of
// the arena and of 16-byte-aligned gradient buffers line up.
struct alignas(32) KvTile {
    int32_t seg;        // segment (key) index in launch order: row of the gradient-pointer table
    int32_t count;      // elements in this tile (<= tile size; the last tile of a key may be ragged)
    int64_t arena_off;  // first element of the tile in the w / m / s arenas (multiple of 4)
    int64_t seg_off;    // first element of the tile inside the key
    int64_t reserved;
};

struct KvLaunchArgs {
    const KvTile* tiles;          // device, all tiles of the store in (unit, key, offset) order
    const void* const* gptrs;     // device, [num_segs * W] gradient pointers, segment-major
    float* w;                     // weight arena
    float* m;                     // momentum arena
    float* s;                     // raw-sum arena (only written by kernels built with KEEP)
    const void* const* bcast;     // device, [num_segs * bcast_n] replica weight pointers, or null
    int32_t bcast_n;              // replicas per key (0 = no broadcast)
    int32_t bcast_f16;            // replicas are fp16 (rounded to nearest even) instead of fp32
    int64_t tile_lo;              // first tile of this launch
    int64_t tile_hi;              // one past the last tile
    int32_t W;
    int32_t xcd_remap;            // G: consecutive tiles per XCD block (0 = tiles dealt one by one)
    int32_t xcd_shift;            // log2(G) if G is a power of two, else -1
    uint32_t xcd_span;            // tiles of the launch rounded up to whole rows of 8 G (the launch's tiles if G = 0)
    uint32_t lds_pad;             // host side only: bytes of LDS each workgroup reserves and never touches, which
                                  // caps the workgroups resident on a compute unit (0 = no cap)
    uint32_t grad_align;          // low 4 bits of the OR of every gradient pointer of the launch's segments: a lane
                                  // width whose vector size divides all of them needs no per-tile alignment check
    float lr, momentum, wd, rescale;
};

// Launch selector: every field picks a template instantiation or a launch shape.
struct KvKernelSel {
    int grad_f16;      // 0: fp32 gradients, 1: fp16
    int W;
    int pairwise;      // 0: rank-order left fold, 1: balanced tree
    int keep_sum;
    int unroll;        // vectors per lane and rank: 1, 2, 4
    int lane_elems;    // consecutive elements per vector: 1, 2, 4
    int nontemporal;
    int generic_w;     // 1: the kernel that takes W at run time, whatever W is
};

// Elements per tile: every lane owns `unroll` vectors of `lane_elems` consecutive elements,
// whatever the gradient dtype.
constexpr int kv_tile_elems(int lane_elems, int unroll) { return KV_THREADS * lane_elems * unroll; }
