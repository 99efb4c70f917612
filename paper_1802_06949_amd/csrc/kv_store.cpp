// C ABI of the key-value gradient aggregation store (see include/kv.h).
//
// Host side of the hot path: records the gradient pointers of every pushed key,
// runs the in-order launch chain and issues ONE fused kernel launch per maximal
// run of consecutive ready units.  The gradient pointers reach the kernel through
// a small device table; tables are cached so that a training loop that reuses its
// gradient buffers (or alternates between a few sets) uploads nothing in steady
// state, and push, pull, wait and barrier allocate no host memory after kv_init
// (tests/native/alloc_count.cpp counts).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "../../include/kv.h"
#include "kv_error.hpp"
#include "kv_kernels.hpp"
#include "kv_plan.hpp"

namespace {

thread_local std::string g_err = "";

void set_err(std::string& dst, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    dst = buf;
}

}  // namespace

void kv_set_global_error(const char* message) { g_err = message ? message : ""; }

namespace {

constexpr int NSLOT = 8;    // cached device pointer tables
constexpr int NSTAGE = 8;   // pinned staging chunks in flight
constexpr int LOG_CAP = 4096;
constexpr int DONE_RING = 256;              // completion events kept for kv_wait(key)
constexpr int DONE_EVERY = 8;               // launches of one stream between two completion events, at most
constexpr int64_t DONE_BYTES = 64LL << 20;  // ... and bytes of launch traffic between two of them, at most

// One cut of the key set into tiles (depends on the elements per tile): the device table, the first
// tile of every unit and of every segment (tiles of segment g: [seg_tile_begin[g], seg_tile_begin[g + 1])).
struct TileSet {
    KvTile* d_tiles = nullptr;
    std::vector<int64_t> unit_tile_begin, seg_tile_begin;
};

// Online tuning (KV_FLAG_AUTOTUNE): every launch shape computes the same bits, so the first
// iterations of a training run can each try another one.  A candidate is timed with a pair of
// events around launches that cover the whole key set; the fastest one is kept.
struct Candidate {
    int lane, cap, xcd;
};
struct Tuner {
    bool active = false;
    int phase = 0;                       // 0: lane width x occupancy cap, 1: XCD block, 2: done
    std::vector<Candidate> cands;
    std::vector<float> best_ms;
    size_t idx = 0;
    int rep = 0;
    bool pending = false;                // a timed launch is in flight
    hipEvent_t e0 = nullptr, e1 = nullptr;
};
constexpr int TUNE_REPS = 2;

struct DoneMark {
    int stream = -1;
    int64_t ordinal = 0;
};

struct Deferred {
    int key;
    void* dst;
    int what;               // 0 = weights, 1 = momentum, 2 = raw sum
};

}  // namespace

struct kv_store {
    kv_plan plan;
    kv_chain chain;
    int W = 0;
    unsigned flags = 0;
    kv_sgd_params p{};
    float rescale = 1.0f;
    int unroll = 1, lane_elems = 4, wg_per_cu = 0, nontemporal = 1, xcd_remap = 0, resident_wgs = 0;
    int generic_w = 0;                            // tuning.run_time_w
    bool wide_ready = false;                      // a second tile table for 4 elements per lane exists (see launch_tiles)
    int64_t wide_launches = 0;
    int tile_elems = 0;
    hipStream_t stream = nullptr;
    int device = 0;
    int num_cus = 256;

    float* w = nullptr;
    float* m = nullptr;
    float* s = nullptr;
    // Tile tables, indexed by log2(lane_elems); only the one in use exists unless the store tunes
    // itself (KV_FLAG_AUTOTUNE).  ts is the one in use.
    TileSet sets[3];
    TileSet* ts = nullptr;
    Tuner tuner;

    size_t table_elems = 0;                       // num_segs * W
    std::vector<const void*> cur_ptrs;            // host: pointers of the pushes not yet launched
    const void** d_slot[NSLOT] = {};
    std::vector<const void*> mirror[NSLOT];       // host copy of what each device table holds
    std::vector<uint8_t> row_valid[NSLOT];        // per segment
    int last_slot = 0;
    int next_victim = 0;

    const void** static_table = nullptr;          // this GPU's file-scope pointer table (kv_push_list_noalloc)
    bool static_call = false;                     // launches of the current call read that table

    const void** h_stage = nullptr;               // pinned, NSTAGE * table_elems
    hipEvent_t stage_ev[NSTAGE] = {};
    bool stage_busy[NSTAGE] = {};
    int stage_next = 0;

    // What kv_wait(key) waits for.  Every launch (or copy) that a key may have to be waited for through gets a
    // mark: the stream it went to (0: the store's, 1 + i: lane i) and its ordinal among that stream's marks.
    // An event record per launch costs about as much host time as the launch itself, so a stream records one
    // only every DONE_EVERY marks, or earlier once DONE_BYTES of traffic have been launched since the last one
    // (a large key gets its own; a run of small ones shares one).  kv_wait(key) waits for the earliest event of
    // the key's stream at or after the key's mark that the ring still holds, else for the stream.
    hipEvent_t done_ev[DONE_RING] = {};
    int done_stream[DONE_RING];
    int64_t done_ordinal[DONE_RING];
    int64_t done_recorded = 0;                    // events recorded so far; the next one goes to slot % DONE_RING
    std::vector<int64_t> marks_issued, marks_at_event, bytes_since_event;   // per stream index
    std::vector<DoneMark> key_mark;               // per key; stream -1: none, wait for the key's stream
    int64_t last_launch_bytes = 0;                // traffic of the launch launch_tiles issued last
    std::vector<uint8_t> want;                    // kv_pull_list: segments asked for (sized at kv_init)

    std::vector<std::vector<Deferred>> deferred;  // per unit
    unsigned capture_mask = 0;                    // iteration being captured: tables that hold every key pushed so far
    bool capture_iteration = false;               // the iteration in progress began inside a capture
    bool capture_launch = false;                  // launches of the current push call are being captured
    bool pinned[NSLOT] = {};                      // read by a captured launch: rows are never overwritten

    // fused broadcast of the updated weights to replica buffers
    int bcast_n = 0;
    int bcast_f16 = 0;
    const void** d_bcast = nullptr;               // device, [num_segs * bcast_n]
    std::vector<const void*> h_bcast;

    float** d_gather = nullptr;                   // device, [num_segs]: destinations of a list pull

    // schedules other than the chained one launch one key at a time
    int schedule = KV_SCHED_CHAINED;
    int outstanding = 0;                          // concurrent schedule: barrier after this many pushes (0 = never)
    int since_barrier = 0;
    std::vector<hipStream_t> lanes;               // concurrent schedule: one stream per "communicator"
    hipEvent_t fork_ev = nullptr;                 // orders a lane after the work already on the main stream
    hipEvent_t join_ev = nullptr;                 // orders the main stream after a lane
    bool in_list = false;                         // inside kv_push_list: one fork event serves the whole list
    bool list_forked = false;
    std::vector<uint8_t> lane_waited;             // per lane: already waits for this list's fork event

    std::vector<std::pair<int, int>> log;
    int64_t launches_total = 0;

    hipEvent_t t0 = nullptr, t1 = nullptr;
    int64_t launches_at_begin = 0;
    bool timing_active = false;
    std::vector<hipEvent_t> marks;               // kv_timing_mark: events between begin and end
    size_t marks_used = 0;

    std::string err;
};

namespace {

#define KV_HIP(store, call)                                                                   \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            set_err((store)->err, "%s failed: %s", #call, hipGetErrorString(e_));             \
            return KV_ERR_HIP;                                                                \
        }                                                                                     \
    } while (0)

void free_store(kv_store* st) {
    if (!st) return;
    if (st->w) (void)hipFree(st->w);
    if (st->m) (void)hipFree(st->m);
    if (st->s) (void)hipFree(st->s);
    for (TileSet& t : st->sets)
        if (t.d_tiles) (void)hipFree(t.d_tiles);
    if (st->tuner.e0) (void)hipEventDestroy(st->tuner.e0);
    if (st->tuner.e1) (void)hipEventDestroy(st->tuner.e1);
    for (int i = 0; i < NSLOT; ++i)
        if (st->d_slot[i]) (void)hipFree(st->d_slot[i]);
    if (st->d_bcast) (void)hipFree(st->d_bcast);
    if (st->d_gather) (void)hipFree(st->d_gather);
    if (st->h_stage) (void)hipHostFree(st->h_stage);
    for (int i = 0; i < NSTAGE; ++i)
        if (st->stage_ev[i]) (void)hipEventDestroy(st->stage_ev[i]);
    for (int i = 0; i < DONE_RING; ++i)
        if (st->done_ev[i]) (void)hipEventDestroy(st->done_ev[i]);
    for (hipStream_t l : st->lanes) (void)hipStreamDestroy(l);
    if (st->fork_ev) (void)hipEventDestroy(st->fork_ev);
    if (st->join_ev) (void)hipEventDestroy(st->join_ev);
    for (hipEvent_t e : st->marks) (void)hipEventDestroy(e);
    if (st->t0) (void)hipEventDestroy(st->t0);
    if (st->t1) (void)hipEventDestroy(st->t1);
    delete st;
}

int check_key(kv_store* st, int key) {
    if (key < 0 || key >= st->plan.num_keys) {
        set_err(st->err, "key %d outside 0..%d", key, st->plan.num_keys - 1);
        return KV_ERR_KEY;
    }
    return KV_OK;
}

// Device table that holds the current pointers of segments [s0, s1); uploads them if
// no cached table matches.
int table_for(kv_store* st, int s0, int s1, hipStream_t stream, const void* const** table_out) {
    const size_t W = (size_t)st->W;
    const size_t lo = (size_t)s0 * W, n = (size_t)(s1 - s0) * W;
    if (st->static_call) {
        // the rows go into the file-scope table by kernel, in stream order before the launch that reads them
        KV_HIP(st, kv_launch_fill_rows(st->static_table, lo, &st->cur_ptrs[lo], n, stream));
        *table_out = st->static_table;
        return KV_OK;
    }
    // A launch that is being captured may only read one of the tables its pushes were checked
    // against, preferably one that an earlier capture already holds; the table is then held too.
    for (int pass = st->capture_launch ? 0 : 1; pass < 2; ++pass) {
        for (int k = 0; k < NSLOT; ++k) {
            const int slot = (st->last_slot + k) % NSLOT;
            if (st->capture_launch && (!(st->capture_mask >> slot & 1u) || (pass == 0 && !st->pinned[slot]))) continue;
            bool valid = true;
            for (int sgm = s0; sgm < s1 && valid; ++sgm) valid = st->row_valid[slot][sgm] != 0;
            if (valid && std::memcmp(&st->mirror[slot][lo], &st->cur_ptrs[lo], n * sizeof(void*)) == 0) {
                if (st->capture_launch) st->pinned[slot] = true;
                st->last_slot = slot;
                *table_out = st->d_slot[slot];
                return KV_OK;
            }
        }
    }
    if (st->capture_launch) {       // unreachable after capture_check; never upload into a capture
        set_err(st->err, "captured launch found no cached pointer table");
        return KV_ERR_STATE;
    }
    // Prefer the table used last if these rows are still free in it (keeps the rows of
    // one iteration together); else evict round robin.
    int slot = st->last_slot;
    bool free_rows = true;
    for (int sgm = s0; sgm < s1 && free_rows; ++sgm) free_rows = st->row_valid[slot][sgm] == 0;
    if (!free_rows) {
        // a table that a captured launch reads is never a victim (at most NSLOT - 1 are pinned)
        slot = st->next_victim;
        for (int tries = 0; tries < NSLOT && (st->pinned[slot] || slot == st->last_slot); ++tries) slot = (slot + 1) % NSLOT;
        if (st->pinned[slot]) slot = st->last_slot;        // every other table is pinned; last_slot then is not
        st->next_victim = (slot + 1) % NSLOT;
    }
    const int chunk = st->stage_next;
    st->stage_next = (st->stage_next + 1) % NSTAGE;
    if (st->stage_busy[chunk]) {
        KV_HIP(st, hipEventSynchronize(st->stage_ev[chunk]));
        st->stage_busy[chunk] = false;
    }
    const void** stage = st->h_stage + (size_t)chunk * st->table_elems + lo;
    std::memcpy(stage, &st->cur_ptrs[lo], n * sizeof(void*));
    KV_HIP(st, hipMemcpyAsync(st->d_slot[slot] + lo, stage, n * sizeof(void*), hipMemcpyHostToDevice, stream));
    KV_HIP(st, hipEventRecord(st->stage_ev[chunk], stream));
    st->stage_busy[chunk] = true;
    std::memcpy(&st->mirror[slot][lo], &st->cur_ptrs[lo], n * sizeof(void*));
    for (int sgm = s0; sgm < s1; ++sgm) st->row_valid[slot][sgm] = 1;
    st->last_slot = slot;
    *table_out = st->d_slot[slot];
    return KV_OK;
}

bool capturing(kv_store* st);

// Gives the work just issued on `stream` (`bytes` of traffic) the stream's next mark, and records a completion
// event when the stream is due one (never called inside a capture: a captured event record is no event the
// host could wait for).
int mark_done(kv_store* st, hipStream_t stream, int64_t bytes, DoneMark* out) {
    int idx = 0;
    for (size_t i = 0; i < st->lanes.size(); ++i)
        if (st->lanes[i] == stream) idx = 1 + (int)i;
    const int64_t ordinal = ++st->marks_issued[(size_t)idx];
    st->bytes_since_event[(size_t)idx] += bytes;
    if (ordinal - st->marks_at_event[(size_t)idx] >= DONE_EVERY || st->bytes_since_event[(size_t)idx] >= DONE_BYTES) {
        const int slot = (int)(st->done_recorded % DONE_RING);
        KV_HIP(st, hipEventRecord(st->done_ev[slot], stream));
        st->done_stream[slot] = idx;
        st->done_ordinal[slot] = ordinal;
        ++st->done_recorded;
        st->marks_at_event[(size_t)idx] = ordinal;
        st->bytes_since_event[(size_t)idx] = 0;
    }
    out->stream = idx;
    out->ordinal = ordinal;
    return KV_OK;
}

int issue_copy_out(kv_store* st, int key, void* dst, int what, hipStream_t stream) {
    const float* base = what == 0 ? st->w : what == 1 ? st->m : st->s;
    const int64_t n = st->plan.numel[key];
    if (n == 0) return KV_OK;
    KV_HIP(st, hipMemcpyAsync(dst, base + st->plan.key_arena_off[key], (size_t)n * sizeof(float), hipMemcpyDefault,
                              stream));
    // kv_wait(key) covers the key's pulls: if the key is waited for through a mark, the copy gets a later one
    if (st->key_mark[(size_t)key].stream >= 0 && !st->capture_launch && !capturing(st)) {
        int rc = mark_done(st, stream, 2 * n * (int64_t)sizeof(float), &st->key_mark[(size_t)key]);
        if (rc != KV_OK) return rc;
    }
    return KV_OK;
}

// One fused kernel launch over the tiles of segments [s0, s1).
//
// Shape of the launch: the store's (one or two elements per lane for 8 and more ranks, ...), except when most of
// the launch's gradient bytes sit in buffers that do not start on a 128-byte line -- views into a flat buffer, say.
// With one element per lane every wavefront's 256-byte piece of such a stream straddles a line that its neighbour
// fetches again (8 fp32 ranks: +7 %, 32 ranks: +21 %, 32 fp16 ranks: +31 %; two elements per lane, 16 ranks: +8 %
// fp32, +11 % fp16); with 4 elements per lane a workgroup covers 4 KB per stream and the shared lines are a quarter
// as many (+3 %, +4 %, +8 %; +4 %, +4 %).  The store keeps a second tile table for that.
int launch_tiles(kv_store* st, int s0, int s1, hipStream_t stream, int log_a, int log_b) {
    if (st->ts->seg_tile_begin[(size_t)s1] <= st->ts->seg_tile_begin[(size_t)s0]) return KV_OK;
    const void* const* table = nullptr;
    int rc = table_for(st, s0, s1, stream, &table);
    if (rc != KV_OK) return rc;
    uintptr_t bits = 0;
    int64_t off_line = 0, total = 0;
    for (int sgm = s0; sgm < s1; ++sgm) {
        uintptr_t row = 0;
        const size_t lo = (size_t)sgm * (size_t)st->W;
        for (size_t i = lo; i < lo + (size_t)st->W; ++i) row |= reinterpret_cast<uintptr_t>(st->cur_ptrs[i]);
        const int64_t n = st->plan.numel[(size_t)st->plan.seg_key[(size_t)sgm]];
        bits |= row;
        total += n;
        if (row & 127u) off_line += n;
    }
    const uintptr_t vec4_mask = (uintptr_t)(4 * st->plan.itemsize - 1);
    const bool wide = st->wide_ready && !st->tuner.active && 2 * off_line > total && (bits & vec4_mask) == 0;
    const TileSet* ts = wide ? &st->sets[2] : st->ts;
    const int64_t tile_lo = ts->seg_tile_begin[(size_t)s0], tile_hi = ts->seg_tile_begin[(size_t)s1];
    if (wide) ++st->wide_launches;
    KvLaunchArgs a{};
    a.tiles = ts->d_tiles;
    a.gptrs = table;
    a.w = st->w;
    a.m = st->m;
    a.s = st->s;
    a.bcast = st->d_bcast;
    a.bcast_n = st->d_bcast ? st->bcast_n : 0;
    a.bcast_f16 = st->bcast_f16;
    a.tile_lo = tile_lo;
    a.tile_hi = tile_hi;
    a.W = st->W;
    a.grad_align = (uint32_t)(bits & 15u);
    // a compute unit has 160 KB of LDS: reserving 160 KB / n per workgroup lets n of them be resident
    a.lds_pad = st->resident_wgs >= 3 && st->resident_wgs < 8 ? (uint32_t)((160 * 1024) / st->resident_wgs) & ~1023u : 0u;
    a.lr = st->p.lr;
    a.momentum = st->p.momentum;
    a.wd = st->p.wd;
    a.rescale = st->rescale;
    KvKernelSel sel{};
    sel.grad_f16 = st->plan.grad_dtype == KV_F16;
    sel.W = st->W;
    sel.pairwise = st->p.reduce_order == KV_REDUCE_PAIRWISE;
    sel.keep_sum = (st->flags & KV_FLAG_KEEP_SUM) != 0;
    sel.unroll = wide ? 1 : st->unroll;
    sel.lane_elems = wide ? 4 : st->lane_elems;
    sel.nontemporal = st->nontemporal;
    sel.generic_w = st->generic_w;
    const int64_t ntiles = tile_hi - tile_lo;
    if (ntiles >= (1LL << 31) - 8 * 4096) {
        set_err(st->err, "a launch of %lld tiles is beyond the kernel's 32-bit tile index", (long long)ntiles);
        return KV_ERR_ARG;
    }
    int64_t span = ntiles;
    a.xcd_remap = 0;
    a.xcd_shift = -1;
    if (st->xcd_remap) {
        // a block never exceeds an eighth of the launch, so a small launch (one key, a small model)
        // does not start workgroups that find no tile
        const int64_t eighth = (ntiles + 7) / 8;
        const int64_t blk = st->xcd_remap == 1 || st->xcd_remap > eighth ? eighth : st->xcd_remap;
        a.xcd_remap = (int32_t)blk;
        for (int sh = 0; sh < 31; ++sh)
            if ((1LL << sh) == blk) a.xcd_shift = sh;
        span = (ntiles + 8 * blk - 1) / (8 * blk) * (8 * blk);
    }
    a.xcd_span = (uint32_t)span;
    int64_t grid = span;
    if (st->wg_per_cu > 0) {
        int64_t cap = (int64_t)st->num_cus * st->wg_per_cu;
        if (st->xcd_remap) cap = (cap + 7) / 8 * 8;
        if (grid > cap) grid = cap;
    }
    if (grid > 0x7FFFFFF0LL) grid = 0x7FFFFFF0LL;       // multiple of 8; the tile loop strides
    KV_HIP(st, kv_launch_fused(sel, a, (unsigned)grid, stream));
    st->last_launch_bytes = total * ((int64_t)st->W * st->plan.itemsize + 4 * (int64_t)sizeof(float));
    if ((int)st->log.size() < LOG_CAP) st->log.emplace_back(log_a, log_b);
    else st->log[(size_t)(st->launches_total % LOG_CAP)] = std::make_pair(log_a, log_b);
    ++st->launches_total;
    return KV_OK;
}

// Launches units [first, first + n) as one kernel, then the pulls queued on them.
void tuner_apply(kv_store* st, const Candidate& c) {
    st->lane_elems = c.lane;
    st->unroll = 1;
    st->tile_elems = kv_tile_elems(c.lane, 1);
    st->ts = &st->sets[c.lane == 1 ? 0 : c.lane == 2 ? 1 : 2];
    st->resident_wgs = c.cap;
    st->xcd_remap = c.xcd;
}

// Called before a launch that covers the whole key set: books the time of the previous timed launch,
// moves on to the next candidate (or locks in the fastest one) and applies it.
int tuner_step(kv_store* st) {
    Tuner& t = st->tuner;
    if (t.pending) {
        float ms = 0.0f;
        KV_HIP(st, hipEventSynchronize(t.e1));
        KV_HIP(st, hipEventElapsedTime(&ms, t.e0, t.e1));
        t.pending = false;
        if (ms < t.best_ms[t.idx]) t.best_ms[t.idx] = ms;
        if (++t.rep >= TUNE_REPS) {
            t.rep = 0;
            ++t.idx;
        }
    }
    if (t.idx >= t.cands.size()) {
        size_t best = 0;
        for (size_t i = 1; i < t.cands.size(); ++i)
            if (t.best_ms[i] < t.best_ms[best]) best = i;
        const Candidate win = t.cands[best];
        const float win_ms = t.best_ms[best];
        if (t.phase == 0) {
            // phase 1: XCD block sizes around the default, for the winning lane width and cap
            t.phase = 1;
            t.cands.clear();                    // capacity stays: no allocation here
            t.best_ms.clear();
            t.cands.push_back(win);
            t.best_ms.push_back(win_ms);
            for (int xcd : {16, 64, 256, 1024})
                if (xcd != win.xcd) {
                    t.cands.push_back(Candidate{win.lane, win.cap, xcd});
                    t.best_ms.push_back(1e30f);
                }
            t.idx = 1;
        } else {
            t.phase = 2;
            t.active = false;
            tuner_apply(st, win);
            return KV_OK;
        }
    }
    tuner_apply(st, t.cands[t.idx]);
    return KV_OK;
}

int launch_run(kv_store* st, int first, int n) {
    const int s0 = st->plan.units[first].seg_begin;
    const int s1 = st->plan.units[first + n - 1].seg_end;
    // a store that tunes itself times the launches that cover the whole key set (never inside a capture)
    const bool timed = st->tuner.active && first == 0 && n == (int)st->plan.units.size() && !st->capture_launch &&
                       !st->capture_iteration;
    if (timed) {
        int rc = tuner_step(st);
        if (rc != KV_OK) return rc;
    }
    const bool record = timed && st->tuner.active;
    if (record) KV_HIP(st, hipEventRecord(st->tuner.e0, st->stream));
    int rc = launch_tiles(st, s0, s1, st->stream, first, n);
    if (rc != KV_OK) return rc;
    if (record) {
        KV_HIP(st, hipEventRecord(st->tuner.e1, st->stream));
        st->tuner.pending = true;
    }
    // kv_wait(key) can wait for this launch through its mark.  A launch that covers the whole key set gets
    // none (one event record per step is measurable on the headline path, and after such a launch waiting for
    // the stream is the same thing); neither does a captured launch.
    DoneMark mk;
    if (n < (int)st->plan.units.size() && !st->capture_launch) {
        rc = mark_done(st, st->stream, st->last_launch_bytes, &mk);
        if (rc != KV_OK) return rc;
    }
    for (int u = first; u < first + n; ++u)
        for (int k : st->plan.units[u].keys) st->key_mark[(size_t)k] = mk;
    for (int u = first; u < first + n; ++u) {
        for (const Deferred& d : st->deferred[u]) {
            rc = issue_copy_out(st, d.key, d.dst, d.what, st->stream);
            if (rc != KV_OK) return rc;
        }
        st->deferred[u].clear();
    }
    return KV_OK;
}

// Stream on which a key's work runs: the store's stream, or in the concurrent schedule the
// lane the key hashes to (key mod number of lanes).
hipStream_t key_stream(const kv_store* st, int key) {
    if (st->schedule == KV_SCHED_CONCURRENT && !st->lanes.empty()) return st->lanes[(size_t)key % st->lanes.size()];
    return st->stream;
}

// Makes a lane wait for everything already issued on the store's stream (the producer of the
// gradients, earlier sets and pulls).  Inside a list push the event is recorded once and every
// lane waits for it once: nothing new can have been issued on the store's stream meanwhile.
int fork_to(kv_store* st, hipStream_t lane, int lane_index) {
    if (lane == st->stream) return KV_OK;
    if (st->in_list) {
        if (!st->list_forked) {
            KV_HIP(st, hipEventRecord(st->fork_ev, st->stream));
            st->list_forked = true;
            std::fill(st->lane_waited.begin(), st->lane_waited.end(), (uint8_t)0);   // sized by kv_set_schedule
        }
        if (lane_index >= 0 && st->lane_waited[(size_t)lane_index]) return KV_OK;
        KV_HIP(st, hipStreamWaitEvent(lane, st->fork_ev, 0));
        if (lane_index >= 0) st->lane_waited[(size_t)lane_index] = 1;
        return KV_OK;
    }
    KV_HIP(st, hipEventRecord(st->fork_ev, st->stream));
    KV_HIP(st, hipStreamWaitEvent(lane, st->fork_ev, 0));
    return KV_OK;
}

int lane_of(const kv_store* st, int key) {
    if (st->schedule == KV_SCHED_CONCURRENT && !st->lanes.empty()) return (int)((size_t)key % st->lanes.size());
    return -1;
}

int barrier_all(kv_store* st) {
    for (hipStream_t l : st->lanes) KV_HIP(st, hipStreamSynchronize(l));
    KV_HIP(st, hipStreamSynchronize(st->stream));
    for (int i = 0; i < NSTAGE; ++i) st->stage_busy[i] = false;
    st->since_barrier = 0;
    return KV_OK;
}

// Funneled and concurrent schedules: the key is launched by its own push.
int launch_key(kv_store* st, int key) {
    const int sgm = st->plan.key_seg[key];
    hipStream_t stream = key_stream(st, key);
    int rc = fork_to(st, stream, lane_of(st, key));
    if (rc != KV_OK) return rc;
    rc = launch_tiles(st, sgm, sgm + 1, stream, key, 0);
    if (rc != KV_OK) return rc;
    st->key_mark[(size_t)key] = DoneMark{};
    if (st->schedule == KV_SCHED_FUNNEL) {
        // the issuing thread does the aggregation itself: nothing else is started before it is done
        KV_HIP(st, hipStreamSynchronize(stream));
        return KV_OK;
    }
    if (!st->capture_launch) {
        rc = mark_done(st, stream, st->last_launch_bytes, &st->key_mark[(size_t)key]);
        if (rc != KV_OK) return rc;
    }
    if (st->outstanding > 0 && ++st->since_barrier >= st->outstanding) {
        return barrier_all(st);
    }
    return KV_OK;
}

int drain_chain(kv_store* st) {
    int first = 0, n = 0;
    while (st->chain.next_run(&first, &n)) {
        int rc = launch_run(st, first, n);
        if (rc != KV_OK) return rc;
    }
    return KV_OK;
}

int check_grads(kv_store* st, int key, const void* const* grads) {
    if (!grads) {
        set_err(st->err, "push of key %d: null gradient pointer array", key);
        return KV_ERR_ARG;
    }
    const uintptr_t mask = (uintptr_t)st->plan.itemsize - 1;
    for (int r = 0; r < st->W; ++r) {
        if (!grads[r] && st->plan.numel[key] > 0) {
            set_err(st->err, "push of key %d: gradient pointer of rank %d is null", key, r);
            return KV_ERR_ARG;
        }
        if ((uintptr_t)grads[r] & mask) {
            set_err(st->err, "push of key %d: gradient pointer of rank %d is not aligned to %d bytes", key, r,
                    st->plan.itemsize);
            return KV_ERR_ALIGN;
        }
    }
    return KV_OK;
}

void record_grads(kv_store* st, int key, const void* const* grads) {
    const size_t row = (size_t)st->plan.key_seg[key] * (size_t)st->W;
    for (int r = 0; r < st->W; ++r) st->cur_ptrs[row + r] = grads[r];
}

// True while the store's stream records into a graph instead of executing.
bool capturing(kv_store* st) {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st->stream, &cs) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return cs == hipStreamCaptureStatusActive;
}

bool row_cached(const kv_store* st, int slot, int key, const void* const* grads) {
    const int sgm = st->plan.key_seg[key];
    if (!st->row_valid[slot][(size_t)sgm]) return false;
    return std::memcmp(&st->mirror[slot][(size_t)sgm * (size_t)st->W], grads, (size_t)st->W * sizeof(void*)) == 0;
}

// While the stream is captured nothing can be uploaded (a recorded copy would read its pinned
// staging chunk again at every replay, long after the chunk has been reused): the pointers of
// every key pushed in the iteration must already sit, together, in a cached device table, i.e. the
// same buffers were pushed before the capture.  capture_mask holds the tables that still qualify.
// Checked before any state changes, so a refused push leaves the store as it was.
int capture_check(kv_store* st, int nkeys, const int* keys, const void* const* grads) {
    if (st->schedule != KV_SCHED_CHAINED) {
        set_err(st->err, "only the chained schedule can be captured into a graph");
        return KV_ERR_STATE;
    }
    const size_t W = (size_t)st->W;
    const bool fresh = st->chain.pending_keys == 0 && st->chain.next_unit == 0;
    if (!fresh && !st->capture_iteration) {
        set_err(st->err, "push while the stream is being captured, but the iteration began before the capture: "
                         "a capture holds whole iterations");
        return KV_ERR_STATE;
    }
    unsigned mask = fresh ? (1u << NSLOT) - 1u : st->capture_mask;
    int bad = -1;
    for (int i = 0; i < nkeys && mask; ++i) {
        unsigned m = 0;
        for (int slot = 0; slot < NSLOT; ++slot)
            if ((mask >> slot & 1u) && row_cached(st, slot, keys[i], grads + (size_t)i * W)) m |= 1u << slot;
        if (!m) bad = keys[i];
        mask = m;
    }
    if (!mask) {
        set_err(st->err, "push of key %d while the stream is being captured: no cached pointer table holds its gradient "
                         "buffers together with those of the keys pushed before it in this iteration (push the same "
                         "buffers once before the capture)", bad);
        return KV_ERR_STATE;
    }
    unsigned pinned_mask = 0;
    int n_pinned = 0;
    for (int slot = 0; slot < NSLOT; ++slot)
        if (st->pinned[slot]) { pinned_mask |= 1u << slot; ++n_pinned; }
    if (!(mask & pinned_mask) && n_pinned >= NSLOT - 1) {
        set_err(st->err, "captured launches already hold %d sets of gradient buffers; kv_release_captures frees them",
                NSLOT - 1);
        return KV_ERR_STATE;
    }
    st->capture_mask = mask;
    st->capture_iteration = true;
    return KV_OK;
}

int pull_common(kv_store* st, int key, void* dst, int what) {
    if (!st) return KV_ERR_ARG;
    int rc = check_key(st, key);
    if (rc != KV_OK) return rc;
    if (!dst && st->plan.numel[key] > 0) {
        set_err(st->err, "pull of key %d: null destination", key);
        return KV_ERR_ARG;
    }
    if (what == 2 && !(st->flags & KV_FLAG_KEEP_SUM)) {
        set_err(st->err, "kv_pull_grad needs a store created with KV_FLAG_KEEP_SUM");
        return KV_ERR_STATE;
    }
    if (st->chain.marked[key] && (st->flags & KV_FLAG_LAZY_LAUNCH)) {
        st->capture_launch = st->capture_iteration && capturing(st);
        rc = drain_chain(st);                  // a pull is a reason to launch what is ready
        st->capture_launch = false;
        if (rc != KV_OK) return rc;
    }
    if (st->chain.marked[key]) {               // pushed, unit not launched yet: run after that launch
        try {
            st->deferred[st->plan.key_unit[key]].push_back(Deferred{key, dst, what});
        } catch (const std::bad_alloc&) {
            set_err(st->err, "out of host memory");
            return KV_ERR_NOMEM;
        }
        return KV_OK;
    }
    hipStream_t stream = key_stream(st, key);
    rc = fork_to(st, stream, lane_of(st, key));
    if (rc != KV_OK) return rc;
    return issue_copy_out(st, key, dst, what, stream);
}

int set_common(kv_store* st, int key, const void* src, float* arena) {
    if (!st) return KV_ERR_ARG;
    int rc = check_key(st, key);
    if (rc != KV_OK) return rc;
    const int64_t n = st->plan.numel[key];
    if (n == 0) return KV_OK;
    if (!src) {
        set_err(st->err, "set of key %d: null source", key);
        return KV_ERR_ARG;
    }
    // The copy always runs on the store's own stream, the one the caller's memory management knows
    // about (a source buffer recycled right after this call must not be read later from another
    // stream).  In the concurrent schedule the store's stream first waits for what the key's lane
    // still has in flight; the key's next launch is ordered after the copy by its fork event.
    hipStream_t lane = key_stream(st, key);
    if (lane != st->stream) {
        KV_HIP(st, hipEventRecord(st->join_ev, lane));
        KV_HIP(st, hipStreamWaitEvent(st->stream, st->join_ev, 0));
    }
    KV_HIP(st, hipMemcpyAsync(arena + st->plan.key_arena_off[key], src, (size_t)n * sizeof(float), hipMemcpyDefault,
                              st->stream));
    return KV_OK;
}

}  // namespace

extern "C" {

// ------------------------------------------------------------------ plan
int kv_plan_create(kv_plan** out, int num_keys, const int64_t* key_numel, int grad_dtype, size_t bucket_bytes) {
    if (!out) {
        set_err(g_err, "kv_plan_create: out is null");
        return KV_ERR_ARG;
    }
    *out = nullptr;
    kv_plan* p = new (std::nothrow) kv_plan();
    if (!p) return KV_ERR_NOMEM;
    int rc = KV_ERR_NOMEM;
    try {
        rc = kv_plan_build(*p, num_keys, key_numel, grad_dtype, bucket_bytes);
    } catch (const std::bad_alloc&) {
        rc = KV_ERR_NOMEM;
    }
    if (rc != KV_OK) {
        set_err(g_err, "kv_plan_create: bad arguments (num_keys=%d, grad_dtype=%d, bucket_bytes=%zu)", num_keys,
                grad_dtype, bucket_bytes);
        delete p;
        return rc;
    }
    *out = p;
    return KV_OK;
}

void kv_plan_destroy(kv_plan* plan) { delete plan; }

int kv_plan_num_keys(const kv_plan* plan) { return plan ? plan->num_keys : KV_ERR_ARG; }
int kv_plan_num_units(const kv_plan* plan) { return plan ? (int)plan->units.size() : KV_ERR_ARG; }

int kv_plan_unit(const kv_plan* plan, int unit, int* is_large_out, int* nkeys_out, int* keys_out, int cap) {
    if (!plan || unit < 0 || unit >= (int)plan->units.size()) return KV_ERR_ARG;
    const KvPlanUnit& u = plan->units[unit];
    if (is_large_out) *is_large_out = u.large ? 1 : 0;
    if (nkeys_out) *nkeys_out = (int)u.keys.size();
    if (keys_out)
        for (int i = 0; i < cap && i < (int)u.keys.size(); ++i) keys_out[i] = u.keys[i];
    return KV_OK;
}

int kv_plan_key(const kv_plan* plan, int key, int* unit_out, int64_t* arena_offset_out) {
    if (!plan) return KV_ERR_ARG;
    if (key < 0 || key >= plan->num_keys) return KV_ERR_KEY;
    if (unit_out) *unit_out = plan->key_unit[key];
    if (arena_offset_out) *arena_offset_out = plan->key_arena_off[key];
    return KV_OK;
}

int64_t kv_plan_arena_numel(const kv_plan* plan) { return plan ? plan->arena_numel : (int64_t)KV_ERR_ARG; }

// ------------------------------------------------------------------ chain
int kv_chain_create(kv_chain** out, const kv_plan* plan) {
    if (!out || !plan) {
        set_err(g_err, "kv_chain_create: null argument");
        return KV_ERR_ARG;
    }
    kv_chain* c = new (std::nothrow) kv_chain();
    if (!c) return KV_ERR_NOMEM;
    c->reset(plan);
    *out = c;
    return KV_OK;
}

void kv_chain_destroy(kv_chain* chain) { delete chain; }
int kv_chain_set_descending(kv_chain* chain, int descending) {
    if (!chain) return KV_ERR_ARG;
    if (chain->pending_keys > 0 || chain->next_unit != 0) return KV_ERR_STATE;
    chain->descending = descending != 0;
    return KV_OK;
}

int kv_chain_mark(kv_chain* chain, int key) { return chain ? chain->mark(key) : KV_ERR_ARG; }

int kv_chain_next_run(kv_chain* chain, int* first_unit_out, int* n_units_out) {
    if (!chain || !first_unit_out || !n_units_out) return KV_ERR_ARG;
    return chain->next_run(first_unit_out, n_units_out) ? 1 : 0;
}

int kv_chain_pending_keys(const kv_chain* chain) { return chain ? chain->pending_keys : KV_ERR_ARG; }
int kv_chain_next_unit(const kv_chain* chain) { return chain ? chain->next_unit : KV_ERR_ARG; }

// ------------------------------------------------------------------ store
int kv_init(kv_store** out, int num_keys, const int64_t* key_numel, int grad_dtype, int W, size_t bucket_bytes,
            const kv_sgd_params* params, unsigned flags, const kv_tuning* tuning, void* hip_stream) {
    if (!out) {
        set_err(g_err, "kv_init: out is null");
        return KV_ERR_ARG;
    }
    *out = nullptr;
    if (!params || W < 1 || W > KV_MAX_W || (flags & ~(unsigned)(KV_FLAG_KEEP_SUM | KV_FLAG_DESCENDING | KV_FLAG_LAZY_LAUNCH | KV_FLAG_AUTOTUNE))) {
        set_err(g_err, "kv_init: bad arguments (params=%p, W=%d, flags=%u)", (const void*)params, W, flags);
        return KV_ERR_ARG;
    }
    if (params->reduce_order != KV_REDUCE_SEQUENTIAL && params->reduce_order != KV_REDUCE_PAIRWISE) {
        set_err(g_err, "kv_init: reduce_order %d unknown", params->reduce_order);
        return KV_ERR_ARG;
    }
    kv_store* st = new (std::nothrow) kv_store();
    if (!st) return KV_ERR_NOMEM;
    int rc = kv_plan_build(st->plan, num_keys, key_numel, grad_dtype, bucket_bytes);
    if (rc != KV_OK) {
        set_err(g_err, "kv_init: bad key set (num_keys=%d, grad_dtype=%d, bucket_bytes=%zu)", num_keys, grad_dtype,
                bucket_bytes);
        delete st;
        return rc;
    }
    st->chain.reset(&st->plan);
    st->chain.descending = (flags & KV_FLAG_DESCENDING) != 0;
    st->W = W;
    st->flags = flags;
    st->p = *params;
    st->rescale = params->rescale > 0.0f ? params->rescale : 1.0f / (float)W;
    st->stream = static_cast<hipStream_t>(hip_stream);

    // Defaults from sweeps on MI355X.  Non-temporal gradient loads keep the streamed gradients
    // from evicting w and m out of the memory-side cache; giving every XCD blocks of consecutive
    // tiles and write-through stores of w', m' are worth a few percent each.
    // State (w and m) that fits the 256 MiB memory-side cache stays resident between iterations
    // if its stores are left to allocate there; state that cannot fit is better streamed past it.
    // Elements per lane: the memory system is fastest when a lane has about 32 bytes of gradients
    // (all W ranks of one vector) in flight, i.e. many small workgroups rather than few large
    // ones; the table holds the measured best width for the rank counts that have a kernel of
    // their own (ResNet-50-shaped key set).
    const int64_t state_bytes = 2 * st->plan.arena_numel * (int64_t)sizeof(float);
    const bool resident = state_bytes <= (256LL << 20);
    // the kernel for any W: measured on the ResNet-50-shaped key set at W = 1, 3, 5, 6, 7, 12, 20, 24, 40, 64
    int lane = grad_dtype == KV_F16 ? (W < 24 ? 4 : W < 36 ? 2 : 1) : (W < 5 ? 4 : W < 18 ? 2 : 1);
    {
        static const int w_built[5] = {2, 4, 8, 16, 32};
        static const int lane_f32[5] = {4, 2, 1, 2, 1};
        static const int lane_f16[5] = {4, 4, 2, 2, 1};
        for (int i = 0; i < 5; ++i)
            if (W == w_built[i]) lane = grad_dtype == KV_F16 ? lane_f16[i] : lane_f32[i];
        // state that is streamed: one element per lane from 16 ranks on, for either dtype
        if (!resident && W == 16) lane = 1;
    }
    // From 16 ranks on even a narrow lane keeps more bytes in flight per compute unit than the memory
    // system likes; fewer resident workgroups are worth another 1-2 %.  When the state does not fit the
    // memory-side cache a cap pays from 2 ranks on (3-8 %; measured on the VGG-16-shaped key set); with
    // resident state and few ranks it costs.
    st->resident_wgs = 0;
    if (grad_dtype == KV_F32) {
        if (W == 16) st->resident_wgs = 4;
        if (W == 32) st->resident_wgs = 4;
        if (W > 32) st->resident_wgs = 5;
        if (!resident && W == 2) st->resident_wgs = 5;
        if (!resident && (W == 4 || W == 8)) st->resident_wgs = 6;
    } else {
        if (resident && W == 16) st->resident_wgs = 5;
        if (!resident && W == 8) st->resident_wgs = 6;
    }
    st->unroll = 1;
    st->lane_elems = lane;
    st->wg_per_cu = 0;
    st->nontemporal = resident ? 9 : 13;
    st->xcd_remap = resident ? 64 : 1024;
    if (tuning) {
        if (tuning->unroll != 0) {
            st->unroll = tuning->unroll;
            st->lane_elems = 4;            // `unroll` alone keeps its meaning of 4-element vectors per lane
        }
        if (tuning->lane_elems != 0) st->lane_elems = tuning->lane_elems;
        if (tuning->workgroups_per_cu >= 0) st->wg_per_cu = tuning->workgroups_per_cu;
        if (tuning->nontemporal >= 0) st->nontemporal = tuning->nontemporal;
        if (tuning->xcd_remap >= 0) st->xcd_remap = tuning->xcd_remap;
        if (tuning->resident_workgroups != 0) st->resident_wgs = tuning->resident_workgroups;
        st->generic_w = tuning->run_time_w;
    }
    const int nt = st->nontemporal;
    const int le = st->lane_elems, un = st->unroll;
    const bool shape_ok = (le == 4 && (un == 1 || un == 2 || un == 4)) || (le == 2 && (un == 1 || un == 2)) ||
                          (le == 1 && (un == 1 || un == 2 || un == 4));
    if (!shape_ok || !(nt == 0 || nt == 1 || nt == 5 || nt == 9 || nt == 13) ||
        !(st->resident_wgs == 0 || (st->resident_wgs >= 3 && st->resident_wgs <= 8)) ||
        st->wg_per_cu > 64 || st->xcd_remap > (1 << 20) || (tuning && tuning->resident_workgroups < 0) ||
        (st->generic_w != 0 && st->generic_w != 1)) {
        set_err(g_err, "kv_init: tuning (lane_elems, unroll) must be one of (4,1) (4,2) (4,4) (2,1) (2,2) (1,1) (1,2) (1,4), "
                       "tuning.nontemporal one of 0, 1, 5, 9, 13, tuning.resident_workgroups 0 or 3..8, "
                       "tuning.workgroups_per_cu at most 64, tuning.xcd_remap at most 2^20 and tuning.run_time_w 0 or 1");
        delete st;
        return KV_ERR_ARG;
    }
    if ((flags & KV_FLAG_AUTOTUNE) && st->unroll != 1) {
        set_err(g_err, "kv_init: KV_FLAG_AUTOTUNE tunes shapes with unroll = 1 only");
        delete st;
        return KV_ERR_ARG;
    }
    st->tile_elems = kv_tile_elems(st->lane_elems, st->unroll);

#define KV_INIT_HIP(call)                                                                     \
    do {                                                                                      \
        hipError_t e_ = (call);                                                               \
        if (e_ != hipSuccess) {                                                               \
            set_err(g_err, "kv_init: %s failed: %s", #call, hipGetErrorString(e_));           \
            free_store(st);                                                                   \
            return KV_ERR_HIP;                                                                \
        }                                                                                     \
    } while (0)

    KV_INIT_HIP(hipGetDevice(&st->device));
    KV_INIT_HIP(kv_static_table(st->device, &st->static_table));
    int cus = 0;
    KV_INIT_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, st->device));
    if (cus > 0) st->num_cus = cus;

    // tile tables: the one of the chosen shape, or one per lane width for a store that tunes itself
    std::vector<KvTile> tiles[3];
    const bool autotune = (flags & KV_FLAG_AUTOTUNE) != 0;
    const int lane_idx = st->lane_elems == 1 ? 0 : st->lane_elems == 2 ? 1 : 2;
    st->ts = &st->sets[lane_idx];
    // a store that runs one element per lane by default (not by the caller's choice), or two with 8 and more ranks,
    // also gets the table for four:
    // launch_tiles switches to it for gradient buffers that are off the 128-byte line grid
    st->wide_ready = (st->lane_elems == 1 || (st->lane_elems == 2 && W >= 8)) && st->unroll == 1 && !(tuning && (tuning->lane_elems != 0 || tuning->unroll != 0));
    const bool build_set[3] = {lane_idx == 0 || autotune, lane_idx == 1 || autotune, lane_idx == 2 || autotune || st->wide_ready};
    try {
        for (int i = 0; i < 3; ++i) {
            if (i == lane_idx) kv_plan_tiles(st->plan, st->tile_elems, tiles[i], st->sets[i].unit_tile_begin, st->sets[i].seg_tile_begin);
            else if (build_set[i]) kv_plan_tiles(st->plan, kv_tile_elems(1 << i, 1), tiles[i], st->sets[i].unit_tile_begin, st->sets[i].seg_tile_begin);
        }
        st->table_elems = st->plan.seg_key.size() * (size_t)W;
        st->cur_ptrs.assign(st->table_elems, nullptr);
        for (int i = 0; i < NSLOT; ++i) {
            st->mirror[i].assign(st->table_elems, nullptr);
            st->row_valid[i].assign(st->plan.seg_key.size(), 0);
        }
        st->deferred.resize(st->plan.units.size());
        for (size_t u = 0; u < st->plan.units.size(); ++u)      // room for a pull of w, m and s per key queued on a unit
            st->deferred[u].reserve(3 * st->plan.units[u].keys.size());
        st->key_mark.assign((size_t)num_keys, DoneMark{});
        st->marks_issued.assign(1 + KV_MAX_STREAMS, 0);
        st->marks_at_event.assign(1 + KV_MAX_STREAMS, 0);
        st->bytes_since_event.assign(1 + KV_MAX_STREAMS, 0);
        st->want.assign(st->plan.seg_key.size(), 0);
        st->log.reserve(LOG_CAP);          // the launch path never allocates
    } catch (const std::bad_alloc&) {
        set_err(g_err, "kv_init: out of host memory");
        free_store(st);
        return KV_ERR_NOMEM;
    }

    const size_t arena_bytes = (size_t)(st->plan.arena_numel > 0 ? st->plan.arena_numel : 4) * sizeof(float);
    KV_INIT_HIP(hipMalloc((void**)&st->w, arena_bytes));
    KV_INIT_HIP(hipMalloc((void**)&st->m, arena_bytes));
    KV_INIT_HIP(hipMemsetAsync(st->w, 0, arena_bytes, st->stream));
    KV_INIT_HIP(hipMemsetAsync(st->m, 0, arena_bytes, st->stream));
    if (flags & KV_FLAG_KEEP_SUM) {
        KV_INIT_HIP(hipMalloc((void**)&st->s, arena_bytes));
        KV_INIT_HIP(hipMemsetAsync(st->s, 0, arena_bytes, st->stream));
    }
    for (int i = 0; i < 3; ++i) {
        if (!build_set[i]) continue;
        const size_t tile_bytes = (tiles[i].empty() ? 1 : tiles[i].size()) * sizeof(KvTile);
        KV_INIT_HIP(hipMalloc((void**)&st->sets[i].d_tiles, tile_bytes));
        if (!tiles[i].empty())
            KV_INIT_HIP(hipMemcpyAsync(st->sets[i].d_tiles, tiles[i].data(), tiles[i].size() * sizeof(KvTile), hipMemcpyHostToDevice,
                                       st->stream));
    }
    if (autotune) {
        KV_INIT_HIP(hipEventCreate(&st->tuner.e0));
        KV_INIT_HIP(hipEventCreate(&st->tuner.e1));
        try {
            // phase 0: lane width x cap of resident workgroups (8 = the hardware's own limit), at the default XCD block
            for (int lane : {1, 2, 4})
                for (int cap : {8, 6, 5, 4}) st->tuner.cands.push_back(Candidate{lane, cap, st->xcd_remap});
            st->tuner.best_ms.assign(st->tuner.cands.size(), 1e30f);
        } catch (const std::bad_alloc&) {
            set_err(g_err, "kv_init: out of host memory");
            free_store(st);
            return KV_ERR_NOMEM;
        }
        st->tuner.active = true;
    }
    for (int i = 0; i < NSLOT; ++i) KV_INIT_HIP(hipMalloc((void**)&st->d_slot[i], st->table_elems * sizeof(void*)));
    KV_INIT_HIP(hipMalloc((void**)&st->d_gather, st->plan.seg_key.size() * sizeof(float*)));
    KV_INIT_HIP(hipHostMalloc((void**)&st->h_stage, (size_t)NSTAGE * st->table_elems * sizeof(void*), hipHostMallocDefault));
    for (int i = 0; i < NSTAGE; ++i) KV_INIT_HIP(hipEventCreateWithFlags(&st->stage_ev[i], hipEventDisableTiming));
    for (int i = 0; i < DONE_RING; ++i) {
        KV_INIT_HIP(hipEventCreateWithFlags(&st->done_ev[i], hipEventDisableTiming));
        st->done_stream[i] = -1;
        st->done_ordinal[i] = 0;
    }
    KV_INIT_HIP(hipEventCreateWithFlags(&st->fork_ev, hipEventDisableTiming));
    KV_INIT_HIP(hipEventCreateWithFlags(&st->join_ev, hipEventDisableTiming));
    KV_INIT_HIP(hipEventCreate(&st->t0));
    KV_INIT_HIP(hipEventCreate(&st->t1));
    // the host vectors `tiles` die at return: wait for their upload
    KV_INIT_HIP(hipStreamSynchronize(st->stream));
#undef KV_INIT_HIP
    *out = st;
    return KV_OK;
}

void kv_destroy(kv_store* store) {
    if (!store) return;
    for (hipStream_t l : store->lanes) (void)hipStreamSynchronize(l);
    (void)hipStreamSynchronize(store->stream);
    free_store(store);
}

int kv_set_weights(kv_store* store, int key, const void* src_f32) {
    return store ? set_common(store, key, src_f32, store->w) : KV_ERR_ARG;
}

int kv_set_momentum(kv_store* store, int key, const void* src_f32) {
    return store ? set_common(store, key, src_f32, store->m) : KV_ERR_ARG;
}

int kv_set_lr(kv_store* store, float lr) {
    if (!store) return KV_ERR_ARG;
    store->p.lr = lr;
    return KV_OK;
}

int kv_set_sgd_params(kv_store* store, const kv_sgd_params* params) {
    if (!store || !params) return KV_ERR_ARG;
    if (params->reduce_order != KV_REDUCE_SEQUENTIAL && params->reduce_order != KV_REDUCE_PAIRWISE) {
        set_err(store->err, "kv_set_sgd_params: reduce_order %d unknown", params->reduce_order);
        return KV_ERR_ARG;
    }
    store->p = *params;
    store->rescale = params->rescale > 0.0f ? params->rescale : 1.0f / (float)store->W;
    return KV_OK;
}

int kv_get_sgd_params(const kv_store* store, kv_sgd_params* params_out) {
    if (!store || !params_out) return KV_ERR_ARG;
    *params_out = store->p;
    params_out->rescale = store->rescale;
    return KV_OK;
}

int kv_push(kv_store* store, int key, const void* const* dev_grads) {
    if (!store) return KV_ERR_ARG;
    int rc = check_key(store, key);
    if (rc != KV_OK) return rc;
    rc = check_grads(store, key, dev_grads);
    if (rc != KV_OK) return rc;
    const bool captured = !store->in_list && capturing(store);
    if (captured) {
        if (store->chain.marked[key]) {
            set_err(store->err, "key %d pushed twice before its unit ran", key);
            return KV_ERR_STATE;
        }
        rc = capture_check(store, 1, &key, dev_grads);
        if (rc != KV_OK) return rc;
    } else if (!store->in_list && store->chain.pending_keys == 0 && store->chain.next_unit == 0) {
        store->capture_iteration = false;
    }
    if (store->schedule != KV_SCHED_CHAINED) {
        record_grads(store, key, dev_grads);
        return launch_key(store, key);
    }
    rc = store->chain.mark(key);
    if (rc != KV_OK) {
        set_err(store->err, "key %d pushed twice before its unit ran", key);
        return rc;
    }
    record_grads(store, key, dev_grads);
    // lazy stores let single pushes pile up until the last key of the iteration is in (then everything
    // that has not run yet goes out as one launch)
    if ((store->flags & KV_FLAG_LAZY_LAUNCH) &&
        store->chain.pending_keys + store->chain.launched_keys < store->plan.num_keys) return KV_OK;
    store->capture_launch = captured;
    rc = drain_chain(store);
    store->capture_launch = false;
    return rc;
}

// Both list pushes.  With static_table the launches read this GPU's file-scope pointer table, filled by
// kernel: nothing is uploaded, so a capture needs no table from an earlier push.
static int push_list_common(kv_store* store, int nkeys, const int* keys, const void* const* dev_grads, bool static_table,
                            const char* fn) {
    if (!store) return KV_ERR_ARG;
    if (nkeys < 0 || (nkeys > 0 && (!keys || !dev_grads))) {
        set_err(store->err, "%s: bad arguments", fn);
        return KV_ERR_ARG;
    }
    if (static_table) {
        if (store->schedule != KV_SCHED_CHAINED) {
            set_err(store->err, "%s: chained schedule only", fn);
            return KV_ERR_STATE;
        }
        if (store->table_elems > (size_t)KV_STATIC_TABLE_PTRS) {
            set_err(store->err, "%s: %zu keys x %d gradient copies = %zu pointers, more than the %d the static table holds",
                    fn, store->plan.seg_key.size(), store->W, store->table_elems, KV_STATIC_TABLE_PTRS);
            return KV_ERR_ARG;
        }
    }
    const bool captured = capturing(store);
    if (captured && store->schedule != KV_SCHED_CHAINED) return capture_check(store, 0, nullptr, nullptr);
    if (store->schedule != KV_SCHED_CHAINED) {
        // keys go out one by one, in list order
        store->in_list = true;
        store->list_forked = false;
        int rc = KV_OK;
        for (int i = 0; i < nkeys && rc == KV_OK; ++i) rc = kv_push(store, keys[i], dev_grads + (size_t)i * store->W);
        store->in_list = false;
        return rc;
    }
    // validate everything before marking anything
    for (int i = 0; i < nkeys; ++i) {
        int rc = check_key(store, keys[i]);
        if (rc != KV_OK) return rc;
        rc = check_grads(store, keys[i], dev_grads + (size_t)i * store->W);
        if (rc != KV_OK) return rc;
        if (store->chain.marked[keys[i]]) {
            set_err(store->err, "key %d pushed twice before its unit ran", keys[i]);
            return KV_ERR_STATE;
        }
    }
    const bool fresh = store->chain.pending_keys == 0 && store->chain.next_unit == 0;
    if (captured && static_table) {
        if (!fresh && !store->capture_iteration) {
            set_err(store->err, "%s while the stream is being captured, but the iteration began before the capture: "
                                "a capture holds whole iterations", fn);
            return KV_ERR_STATE;
        }
        if (fresh) store->capture_mask = 0;            // no cached table is known to hold this iteration
        store->capture_iteration = true;
    } else if (captured) {
        int rc = capture_check(store, nkeys, keys, dev_grads);
        if (rc != KV_OK) return rc;
    } else if (fresh) {
        store->capture_iteration = false;
    }
    for (int i = 0; i < nkeys; ++i) {
        if (store->chain.mark(keys[i]) != KV_OK) {          // duplicate inside the list: undo
            for (int j = 0; j < i; ++j) {
                store->chain.marked[keys[j]] = 0;
                ++store->chain.pending[store->plan.key_unit[keys[j]]];
                --store->chain.pending_keys;
            }
            set_err(store->err, "key %d appears twice in one push list", keys[i]);
            return KV_ERR_STATE;
        }
    }
    for (int i = 0; i < nkeys; ++i) record_grads(store, keys[i], dev_grads + (size_t)i * store->W);
    store->capture_launch = captured;
    store->static_call = static_table;
    const int rc = drain_chain(store);
    store->static_call = false;
    store->capture_launch = false;
    return rc;
}

int kv_push_list(kv_store* store, int nkeys, const int* keys, const void* const* dev_grads) {
    return push_list_common(store, nkeys, keys, dev_grads, false, "kv_push_list");
}

int kv_push_list_noalloc(kv_store* store, int nkeys, const int* keys, const void* const* dev_grads) {
    return push_list_common(store, nkeys, keys, dev_grads, true, "kv_push_list_noalloc");
}

int kv_pull(kv_store* store, int key, void* dev_out_f32) { return pull_common(store, key, dev_out_f32, 0); }
int kv_pull_momentum(kv_store* store, int key, void* dev_out_f32) { return pull_common(store, key, dev_out_f32, 1); }
int kv_pull_grad(kv_store* store, int key, void* dev_out_f32) { return pull_common(store, key, dev_out_f32, 2); }

int kv_pull_list(kv_store* store, int nkeys, const int* keys, void* const* dev_out_f32) {
    if (!store) return KV_ERR_ARG;
    if (nkeys < 0 || (nkeys > 0 && (!keys || !dev_out_f32))) {
        set_err(store->err, "kv_pull_list: bad arguments");
        return KV_ERR_ARG;
    }
    const size_t nseg = store->plan.seg_key.size();
    // The gather reads a table of destinations that is uploaded from a reusable pinned chunk: a capture would
    // re-read that chunk at every replay, long after it holds something else.  Under capture (and in the
    // concurrent schedule) the list is served key by key with device-to-device copies instead.
    bool simple = store->schedule != KV_SCHED_CONCURRENT && !capturing(store);
    std::vector<uint8_t>& want = store->want;
    std::fill(want.begin(), want.end(), (uint8_t)0);
    for (int i = 0; i < nkeys; ++i) {
        int rc = check_key(store, keys[i]);
        if (rc != KV_OK) return rc;
        if (!dev_out_f32[i] && store->plan.numel[keys[i]] > 0) {
            set_err(store->err, "kv_pull_list: null destination for key %d", keys[i]);
            return KV_ERR_ARG;
        }
        if ((uintptr_t)dev_out_f32[i] & 3u) {
            set_err(store->err, "kv_pull_list: destination of key %d is not aligned to 4 bytes", keys[i]);
            return KV_ERR_ALIGN;
        }
        const int sgm = store->plan.key_seg[keys[i]];
        if (store->chain.marked[keys[i]] || want[(size_t)sgm]) simple = false;    // pending push, or listed twice
        want[(size_t)sgm] = 1;
    }
    if (!simple) {                      // one by one: queued behind pending launches, or on the keys' own streams
        for (int i = 0; i < nkeys; ++i) {
            int rc = pull_common(store, keys[i], dev_out_f32[i], 0);
            if (rc != KV_OK) return rc;
        }
        return KV_OK;
    }
    // destinations go to the device through a pinned staging chunk, then one gather per run of
    // consecutive segments
    const int chunk = store->stage_next;
    store->stage_next = (store->stage_next + 1) % NSTAGE;
    if (store->stage_busy[chunk]) {
        KV_HIP(store, hipEventSynchronize(store->stage_ev[chunk]));
        store->stage_busy[chunk] = false;
    }
    const void** stage = store->h_stage + (size_t)chunk * store->table_elems;     // table_elems >= nseg
    for (size_t sgm = 0; sgm < nseg; ++sgm) stage[sgm] = nullptr;
    for (int i = 0; i < nkeys; ++i) stage[(size_t)store->plan.key_seg[keys[i]]] = dev_out_f32[i];
    KV_HIP(store, hipMemcpyAsync(store->d_gather, stage, nseg * sizeof(float*), hipMemcpyHostToDevice, store->stream));
    KV_HIP(store, hipEventRecord(store->stage_ev[chunk], store->stream));
    store->stage_busy[chunk] = true;
    for (size_t a = 0; a < nseg;) {
        if (!want[a]) { ++a; continue; }
        size_t b = a;
        while (b < nseg && want[b]) ++b;
        KV_HIP(store, kv_launch_gather(store->ts->d_tiles, store->ts->seg_tile_begin[a], store->ts->seg_tile_begin[b], store->w,
                                       store->d_gather, store->stream));
        a = b;
    }
    // kv_wait(key) covers the key's pulls: keys waited for through a mark get the mark of the gather
    DoneMark mk;
    for (int i = 0; i < nkeys; ++i) {
        if (store->key_mark[(size_t)keys[i]].stream < 0) continue;
        if (mk.stream < 0) {
            int64_t bytes = 0;
            for (int j = 0; j < nkeys; ++j) bytes += 2 * store->plan.numel[(size_t)keys[j]] * (int64_t)sizeof(float);
            int rc = mark_done(store, store->stream, bytes, &mk);
            if (rc != KV_OK) return rc;
        }
        store->key_mark[(size_t)keys[i]] = mk;
    }
    return KV_OK;
}

int kv_weights_ptr(kv_store* store, int key, void** dev_ptr_out) {
    if (!store || !dev_ptr_out) return KV_ERR_ARG;
    int rc = check_key(store, key);
    if (rc != KV_OK) return rc;
    *dev_ptr_out = store->w + store->plan.key_arena_off[key];
    return KV_OK;
}

int kv_wait(kv_store* store, int key) {
    if (!store) return KV_ERR_ARG;
    if ((store->flags & KV_FLAG_LAZY_LAUNCH) && store->schedule == KV_SCHED_CHAINED) {
        int rc = drain_chain(store);
        if (rc != KV_OK) return rc;
    }
    if (key >= 0) {
        int rc = check_key(store, key);
        if (rc != KV_OK) return rc;
        if (store->chain.marked[key]) {
            set_err(store->err, "kv_wait: key %d is pushed but its unit waits for other keys or lower units", key);
            return KV_ERR_INCOMPLETE;
        }
        // the earliest event held that the key's stream recorded at or after the key's last launch (or a pull
        // issued after it); without one (the stream has issued fewer than DONE_EVERY marks since) the stream
        const DoneMark mk = store->key_mark[(size_t)key];
        int best = -1;
        if (mk.stream >= 0) {
            const int held = store->done_recorded < DONE_RING ? (int)store->done_recorded : DONE_RING;
            for (int i = 0; i < held; ++i)
                if (store->done_stream[i] == mk.stream && store->done_ordinal[i] >= mk.ordinal &&
                    (best < 0 || store->done_ordinal[i] < store->done_ordinal[best]))
                    best = i;
        }
        if (best >= 0) KV_HIP(store, hipEventSynchronize(store->done_ev[best]));
        else KV_HIP(store, hipStreamSynchronize(key_stream(store, key)));
        return KV_OK;
    }
    if (key != -1) {
        set_err(store->err, "kv_wait: key %d", key);
        return KV_ERR_KEY;
    }
    {
        int rc = barrier_all(store);
        if (rc != KV_OK) return rc;
    }
    if (store->chain.pending_keys > 0 || store->chain.next_unit != 0) {
        set_err(store->err, "kv_wait: iteration incomplete (%d keys pushed but not launched, next unit %d)",
                store->chain.pending_keys, store->chain.next_unit);
        return KV_ERR_INCOMPLETE;
    }
    return KV_OK;
}

int kv_set_broadcast(kv_store* store, int key, int n_replicas, void* const* dev_dst, int dtype) {
    if (!store) return KV_ERR_ARG;
    int rc = check_key(store, key);
    if (rc != KV_OK) return rc;
    if (n_replicas < 0 || n_replicas > KV_MAX_W || (n_replicas > 0 && !dev_dst) || (dtype != KV_F32 && dtype != KV_F16)) {
        set_err(store->err, "kv_set_broadcast: bad arguments (n_replicas=%d, dtype=%d)", n_replicas, dtype);
        return KV_ERR_ARG;
    }
    if (store->chain.marked[key]) {
        set_err(store->err, "kv_set_broadcast: key %d is pushed and waits for its launch", key);
        return KV_ERR_STATE;
    }
    if (n_replicas == 0 && store->bcast_n == 0) return KV_OK;
    if (store->bcast_n != 0 && n_replicas != 0 && (n_replicas != store->bcast_n || (dtype == KV_F16) != (store->bcast_f16 != 0))) {
        set_err(store->err, "kv_set_broadcast: every key of a store uses the same replica count and dtype (%d, %s)",
                store->bcast_n, store->bcast_f16 ? "f16" : "f32");
        return KV_ERR_STATE;
    }
    const uintptr_t mask = dtype == KV_F16 ? 1u : 3u;
    for (int r = 0; r < n_replicas; ++r) {
        if (!dev_dst[r] && store->plan.numel[key] > 0) {
            set_err(store->err, "kv_set_broadcast: replica pointer %d of key %d is null", r, key);
            return KV_ERR_ARG;
        }
        if ((uintptr_t)dev_dst[r] & mask) {
            set_err(store->err, "kv_set_broadcast: replica pointer %d of key %d is not aligned to its element", r, key);
            return KV_ERR_ALIGN;
        }
    }
    // launches in flight may be reading the table
    rc = barrier_all(store);
    if (rc != KV_OK) return rc;
    const size_t nseg = store->plan.seg_key.size();
    if (store->bcast_n == 0) {
        try {
            store->h_bcast.assign(nseg * (size_t)n_replicas, nullptr);
        } catch (const std::bad_alloc&) {
            return KV_ERR_NOMEM;
        }
        KV_HIP(store, hipMalloc((void**)&store->d_bcast, store->h_bcast.size() * sizeof(void*)));
        KV_HIP(store, hipMemset(store->d_bcast, 0, store->h_bcast.size() * sizeof(void*)));
        store->bcast_n = n_replicas;
        store->bcast_f16 = dtype == KV_F16;
    }
    const size_t row = (size_t)store->plan.key_seg[key] * (size_t)store->bcast_n;
    // a key with no elements keeps a null row: it has no tiles, the kernel never looks at it
    for (int r = 0; r < store->bcast_n; ++r)
        store->h_bcast[row + r] = (n_replicas > 0 && store->plan.numel[key] > 0) ? dev_dst[r] : nullptr;
    KV_HIP(store, hipMemcpy(store->d_bcast + row, &store->h_bcast[row], (size_t)store->bcast_n * sizeof(void*),
                            hipMemcpyHostToDevice));
    return KV_OK;
}

int kv_broadcast_weights(kv_store* store, int key) {
    if (!store) return KV_ERR_ARG;
    if (key != -1) {
        int rc = check_key(store, key);
        if (rc != KV_OK) return rc;
    }
    if (store->bcast_n == 0 || !store->d_bcast) return KV_OK;           // no key has replicas
    const int k0 = key == -1 ? 0 : key, k1 = key == -1 ? store->plan.num_keys : key + 1;
    for (int k = k0; k < k1; ++k) {
        if (store->chain.marked[k]) {
            set_err(store->err, "kv_broadcast_weights: key %d is pushed and waits for its launch", k);
            return KV_ERR_STATE;
        }
    }
    if (key == -1 && store->schedule != KV_SCHED_CONCURRENT) {
        // segments are in arena order: all keys are one contiguous range of tiles
        const size_t nseg = store->plan.seg_key.size();
        KV_HIP(store, kv_launch_replicate(store->ts->d_tiles, store->ts->seg_tile_begin[0], store->ts->seg_tile_begin[nseg], store->w,
                                          store->d_bcast, store->bcast_n, store->bcast_f16, store->stream));
        return KV_OK;
    }
    for (int k = k0; k < k1; ++k) {
        const int sgm = store->plan.key_seg[k];
        hipStream_t stream = key_stream(store, k);
        int rc = fork_to(store, stream, lane_of(store, k));
        if (rc != KV_OK) return rc;
        KV_HIP(store, kv_launch_replicate(store->ts->d_tiles, store->ts->seg_tile_begin[sgm], store->ts->seg_tile_begin[sgm + 1],
                                          store->w, store->d_bcast, store->bcast_n, store->bcast_f16, stream));
    }
    return KV_OK;
}

int kv_get_tuning(const kv_store* store, kv_tuning* tuning_out, int* tuning_done_out) {
    if (!store || !tuning_out) return KV_ERR_ARG;
    tuning_out->unroll = store->unroll;
    tuning_out->workgroups_per_cu = store->wg_per_cu;
    tuning_out->nontemporal = store->nontemporal;
    tuning_out->xcd_remap = store->xcd_remap;
    tuning_out->lane_elems = store->lane_elems;
    tuning_out->resident_workgroups = store->resident_wgs;
    tuning_out->run_time_w = store->generic_w;
    if (tuning_done_out) *tuning_done_out = store->tuner.active ? 0 : 1;
    return KV_OK;
}

int kv_wide_launches(const kv_store* store, int64_t* count_out) {
    if (!store || !count_out) return KV_ERR_ARG;
    *count_out = store->wide_launches;
    return KV_OK;
}

int kv_completion_events(const kv_store* store, int64_t* count_out) {
    if (!store || !count_out) return KV_ERR_ARG;
    *count_out = store->done_recorded;
    return KV_OK;
}

int kv_release_captures(kv_store* store) {
    if (!store) return KV_ERR_ARG;
    for (int i = 0; i < NSLOT; ++i) store->pinned[i] = false;
    store->capture_mask = 0;
    return KV_OK;
}

int kv_wait_event(kv_store* store, void* hip_event) {
    if (!store || !hip_event) return KV_ERR_ARG;
    KV_HIP(store, hipStreamWaitEvent(store->stream, static_cast<hipEvent_t>(hip_event), 0));
    return KV_OK;
}

int kv_barrier(kv_store* store) {
    if (!store) return KV_ERR_ARG;
    if ((store->flags & KV_FLAG_LAZY_LAUNCH) && store->schedule == KV_SCHED_CHAINED) {
        int rc = drain_chain(store);
        if (rc != KV_OK) return rc;
    }
    return barrier_all(store);
}

int kv_set_schedule(kv_store* store, int schedule, int n_streams, int outstanding) {
    if (!store) return KV_ERR_ARG;
    if (schedule != KV_SCHED_CHAINED && schedule != KV_SCHED_FUNNEL && schedule != KV_SCHED_CONCURRENT) {
        set_err(store->err, "kv_set_schedule: unknown schedule %d", schedule);
        return KV_ERR_ARG;
    }
    if (schedule == KV_SCHED_CONCURRENT && (n_streams < 1 || n_streams > KV_MAX_STREAMS || outstanding < 0)) {
        set_err(store->err, "kv_set_schedule: n_streams must be 1..%d and outstanding >= 0", KV_MAX_STREAMS);
        return KV_ERR_ARG;
    }
    if (store->chain.pending_keys > 0 || store->chain.next_unit != 0) {
        set_err(store->err, "kv_set_schedule: an iteration is in progress");
        return KV_ERR_STATE;
    }
    int rc = barrier_all(store);
    if (rc != KV_OK) return rc;
    if (schedule == KV_SCHED_CONCURRENT) {
        try {
            while ((int)store->lanes.size() < n_streams) {
                hipStream_t l = nullptr;
                KV_HIP(store, hipStreamCreateWithFlags(&l, hipStreamNonBlocking));     // default priority
                store->lanes.push_back(l);
            }
            store->lane_waited.assign((size_t)n_streams, 0);
        } catch (const std::bad_alloc&) {
            return KV_ERR_NOMEM;
        }
        while ((int)store->lanes.size() > n_streams) {
            (void)hipStreamDestroy(store->lanes.back());
            store->lanes.pop_back();
        }
        store->lane_waited.resize(store->lanes.size());
        store->outstanding = outstanding;
    } else {
        store->outstanding = 0;
    }
    store->since_barrier = 0;
    store->schedule = schedule;
    // everything is complete, and a key's stream may be another one from here on
    for (DoneMark& mk : store->key_mark) mk = DoneMark{};
    return KV_OK;
}

const kv_plan* kv_store_plan(const kv_store* store) { return store ? &store->plan : nullptr; }

int kv_launch_log(const kv_store* store, int64_t* total_out, int* first_unit_out, int* n_units_out, int cap) {
    if (!store) return KV_ERR_ARG;
    if (total_out) *total_out = store->launches_total;
    if (cap <= 0 || !first_unit_out || !n_units_out) return KV_OK;
    const int64_t have = (int64_t)store->log.size();
    int64_t n = have < cap ? have : cap;
    for (int64_t i = 0; i < n; ++i) {
        const int64_t idx = store->launches_total - n + i;          // absolute launch number
        const auto& e = store->log[(size_t)(idx % LOG_CAP)];
        first_unit_out[i] = e.first;
        n_units_out[i] = e.second;
    }
    return (int)n;
}

int kv_timing_begin(kv_store* store) {
    if (!store) return KV_ERR_ARG;
    KV_HIP(store, hipEventRecord(store->t0, store->stream));
    store->launches_at_begin = store->launches_total;
    store->timing_active = true;
    store->marks_used = 0;
    return KV_OK;
}

int kv_timing_mark(kv_store* store) {
    if (!store) return KV_ERR_ARG;
    if (!store->timing_active) {
        set_err(store->err, "kv_timing_mark without kv_timing_begin");
        return KV_ERR_STATE;
    }
    if (store->marks_used == store->marks.size()) {
        if (store->marks.size() >= (size_t)KV_MAX_TIMING_MARKS) {
            set_err(store->err, "kv_timing_mark: more than %d marks", KV_MAX_TIMING_MARKS);
            return KV_ERR_STATE;
        }
        hipEvent_t e = nullptr;
        KV_HIP(store, hipEventCreate(&e));
        try {
            store->marks.push_back(e);
        } catch (const std::bad_alloc&) {
            (void)hipEventDestroy(e);
            return KV_ERR_NOMEM;
        }
    }
    KV_HIP(store, hipEventRecord(store->marks[store->marks_used], store->stream));
    ++store->marks_used;
    return KV_OK;
}

int kv_timing_intervals(kv_store* store, float* ms_out, int cap) {
    if (!store || (cap > 0 && !ms_out)) return KV_ERR_ARG;
    if (store->timing_active) {
        set_err(store->err, "kv_timing_intervals before kv_timing_end");
        return KV_ERR_STATE;
    }
    int n = 0;
    hipEvent_t prev = store->t0;
    for (size_t i = 0; i < store->marks_used && n < cap; ++i, ++n) {
        KV_HIP(store, hipEventElapsedTime(&ms_out[n], prev, store->marks[i]));
        prev = store->marks[i];
    }
    return n;
}

int kv_timing_end(kv_store* store, float* ms_out, int64_t* launches_out) {
    if (!store || !ms_out) return KV_ERR_ARG;
    if (!store->timing_active) {
        set_err(store->err, "kv_timing_end without kv_timing_begin");
        return KV_ERR_STATE;
    }
    KV_HIP(store, hipEventRecord(store->t1, store->stream));
    KV_HIP(store, hipEventSynchronize(store->t1));
    KV_HIP(store, hipEventElapsedTime(ms_out, store->t0, store->t1));
    if (launches_out) *launches_out = store->launches_total - store->launches_at_begin;
    store->timing_active = false;
    return KV_OK;
}

const char* kv_last_error(const kv_store* store) { return store ? store->err.c_str() : g_err.c_str(); }

}  // extern "C"
