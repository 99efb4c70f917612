/*
 * kv.h - C ABI of the MI355X key-value gradient aggregation library.
 *
 * The library implements, on ONE GPU, the push / pull problem of the paper's
 * "KVStore API" section: every parameter tensor has an integer key; push hands
 * over the gradient copies of a key, which are aggregated (summed over the W
 * workers); pull returns the value for the key.  Here the W workers' gradient
 * copies already sit in this GPU's memory, the aggregate is multiplied by a
 * scaling factor ("Parallel SGD" section) and the weight update of eq. (1),
 * extended by momentum and L2 weight decay, is applied in the same kernel:
 *
 *     s     = g_0 + g_1 + ... + g_{W-1}          (fp32; order: see kv_sgd_params)
 *     ghat  = rescale * s
 *     dw    = momentum * m - lr * (ghat + wd * w)
 *     w'    = w + dw,   m' = dw                   (eq. (1): w_{t+1} = w_t + dw)
 *
 * Every operation is IEEE binary32 with one rounding (no fused multiply-add),
 * subnormals are kept; half-precision gradients are widened exactly first.
 *
 * Scheduling follows the paper's "MPI Dependency Chaining" design: keys smaller
 * than bucket_bytes are packed into buckets, every bucket or large key is a
 * "unit", and units are launched strictly in ascending unit index whatever
 * order the pushes arrive in (the paper orders its collectives with a dummy
 * write dependency; here the order is a function of the key set alone).
 *
 * Conventions
 *   - All functions return KV_OK (0) or a negative kv_status; none throws or
 *     aborts.  kv_last_error() gives a message for the last failure.
 *   - "dev" pointers are device memory of the GPU that was current at kv_init;
 *     "host" pointers are ordinary host memory.  Nothing passed in is freed by
 *     the library; everything the library allocates is freed by kv_destroy.
 *   - A store is not thread-safe: one issuing thread (as in the paper, where
 *     only the main thread issues engine operations).
 *   - All device work is issued on the HIP stream given to kv_init.
 */
#ifndef KV_H
#define KV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kv_store kv_store;   /* opaque, library-owned */
typedef struct kv_plan  kv_plan;    /* opaque, host-only bucket plan */
typedef struct kv_chain kv_chain;   /* opaque, host-only launch-order state machine */

enum kv_status {
    KV_OK             =  0,
    KV_ERR_ARG        = -1,   /* null pointer, bad count, bad enum value            */
    KV_ERR_KEY        = -2,   /* key id outside 0..num_keys-1                        */
    KV_ERR_STATE      = -3,   /* second push of a key before its unit ran; feature off */
    KV_ERR_ALIGN      = -4,   /* gradient pointer not aligned to its element size    */
    KV_ERR_INCOMPLETE = -5,   /* wait / barrier while pushed keys cannot be launched  */
    KV_ERR_HIP        = -6,   /* a HIP runtime call failed (no device, out of memory) */
    KV_ERR_NOMEM      = -7    /* host allocation failed                              */
};

enum kv_dtype { KV_F32 = 0, KV_F16 = 1 };                 /* gradient element type   */
enum kv_reduce_order { KV_REDUCE_SEQUENTIAL = 0,          /* s = g_0; s += g_r, r=1.. */
                       KV_REDUCE_PAIRWISE   = 1 };        /* balanced tree, see below */
enum kv_flags { KV_FLAG_KEEP_SUM   = 1u,                  /* also store s (kv_pull_grad) */
                KV_FLAG_DESCENDING = 2u,                  /* units run from the last one down to unit 0: the
                                                             order in which a backward pass produces gradients
                                                             (last layer first).  Still a function of the key
                                                             set alone, so the same on every worker. */
                KV_FLAG_LAZY_LAUNCH = 4u,               /* a single kv_push launches nothing until every key
                                                             of the iteration is pushed (then all units go out
                                                             as ONE launch), or until a pull, wait or barrier
                                                             asks for what is ready: the paper's Dependency
                                                             Chaining loop, which issues all pushes before the
                                                             first pull */
                KV_FLAG_AUTOTUNE = 8u };                  /* the store tunes its launch shape while it runs: every
                                                             shape computes the same bits, so the first ~35
                                                             launches that cover the whole key set (list pushes of
                                                             all keys, or a lazy store) each try another lane
                                                             width, cap of resident workgroups or XCD block, timed
                                                             with events; the fastest is kept (kv_get_tuning).  Each
                                                             trial waits for the previous launch on the host.
                                                             Needs unroll = 1; never runs inside a graph capture */

/*
 * The paper's three ways of embedding the aggregation into the worker's task flow
 * (section "Embedding MPI operators in DAGs").  All three compute the same values.
 *   KV_SCHED_CHAINED     "MPI Dependency Chaining": pushes only record; units are launched in one
 *                        fixed order, merged, without ever blocking the issuing thread.  Default.
 *   KV_SCHED_FUNNEL      "MPI Funneled": the issuing thread does the aggregation of a key itself, in
 *                        its push, and nothing else starts before it is done: one key per launch,
 *                        no buckets (the paper keeps one communication buffer per key), the host
 *                        blocks until the launch has completed, so one aggregation is outstanding.
 *   KV_SCHED_CONCURRENT  "MPI Concurrent Communications": several communicators, here HIP streams;
 *                        a key is hashed to stream (key mod n_streams) and launched there by its
 *                        push without blocking; after every `outstanding` pushes (0 = never) the
 *                        store runs kv_barrier, as the paper's Python loop does every OUTSTANDING keys.
 */
enum kv_schedule { KV_SCHED_CHAINED = 0, KV_SCHED_FUNNEL = 1, KV_SCHED_CONCURRENT = 2 };

#define KV_MAX_W 256
#define KV_MAX_STREAMS 64
#define KV_MAX_TIMING_MARKS 8192

/*
 * Optimizer parameters.  rescale <= 0 selects 1.0f / (float)W, computed once in
 * fp32 and multiplied.  reduce_order PAIRWISE sums ranks as the tree
 * sum(lo,1) = g_lo; sum(lo,n) = sum(lo,h) + sum(lo+h, n-h), h the largest
 * power of two strictly below n.  The first term of SEQUENTIAL is g_0 itself.
 */
typedef struct kv_sgd_params {
    float lr;
    float momentum;
    float wd;
    float rescale;
    int   reduce_order;
} kv_sgd_params;

/*
 * Launch tuning; pass NULL for defaults.  None of these changes any result bit.
 *   unroll            vectors per thread per rank in one tile: 1, 2 or 4 (0 = default)
 *   lane_elems        consecutive elements per vector, i.e. per thread and load instruction: 1, 2 or 4
 *                     (0 = default: chosen from W and the gradient dtype, or 4 if unroll is given); a tile
 *                     is 256 * lane_elems * unroll elements; (lane_elems, unroll) must be one of
 *                     (4,1) (4,2) (4,4) (2,1) (2,2) (1,1) (1,2) (1,4)
 *   workgroups_per_cu cap of resident workgroups per compute unit for the grid-stride
 *                     loop over tiles, 1..64; 0 = one workgroup per tile; negative = default (0)
 *   nontemporal       cache policy: bit 0 = gradient loads carry the non-temporal hint; plus the policy
 *                     of the stores of w', m' (and s): 0 = plain, 4 = non-temporal, 8 = write through L2,
 *                     12 = write through L2 and non-temporal; one of 0, 1, 5, 9, 13; -1 = default (9 if
 *                     w and m together fit the 256 MiB memory-side cache, else 13)
 *   resident_workgroups  cap of workgroups resident per compute unit, 3..7, enforced by reserving LDS; 8 = no
 *                     cap (the hardware's own limit for workgroups of 256 lanes); 0 = default (a cap for 16 or 32 fp32 ranks, and for most rank
 *                     counts when w and m do not fit the memory-side cache).  Unlike
 *                     workgroups_per_cu the grid still has one workgroup per tile.
 *   xcd_remap         how tiles are dealt to the 8 XCDs: 0 = one by one, round robin; 1 = eight contiguous
 *                     ranges, one per XCD (so a block of one tile cannot be asked for; 0 deals single tiles);
 *                     G = 2..2^20 = blocks of G consecutive tiles per XCD, never more than an eighth of a launch;
 *                     negative = default (64, or 1024 if w and m do not fit the memory-side cache)
 *   run_time_w        1 = run the kernel that takes W at run time even where a kernel built for this W exists
 *                     (W = 2, 4, 8, 16, 32); 0 = default.  For measuring one against the other and for tests.
 * Values outside these ranges make kv_init fail with KV_ERR_ARG; kv_get_tuning returns the values in force.
 */
typedef struct kv_tuning {
    int unroll;
    int workgroups_per_cu;
    int nontemporal;
    int xcd_remap;
    int lane_elems;
    int resident_workgroups;
    int run_time_w;
} kv_tuning;

/* ------------------------------------------------------------------ plan (host only)
 * The bucket plan is a pure function of (key_numel[], grad_dtype, bucket_bytes);
 * it needs no GPU.  Policy (the paper has one communication buffer per key and no
 * buckets; this is this library's extension): scan keys in ascending id; a key's
 * size is numel * sizeof(grad element) of ONE copy; size >= bucket_bytes makes the
 * key a unit of its own ("large") and leaves the open bucket open; a smaller key
 * joins the open bucket if the bucket stays <= bucket_bytes, else closes it and
 * opens a new one.  Units are numbered by the id of their first key.  In the
 * weight / momentum arena units lie in index order, keys ascending inside a unit,
 * every key start rounded up to 256 bytes (64 fp32 elements).
 */
int     kv_plan_create(kv_plan** out, int num_keys, const int64_t* key_numel /* host [num_keys], each >= 0 */,
                       int grad_dtype, size_t bucket_bytes /* >= 1 */);
void    kv_plan_destroy(kv_plan* plan);
int     kv_plan_num_keys(const kv_plan* plan);                 /* < 0 on NULL */
int     kv_plan_num_units(const kv_plan* plan);
/* Unit description.  keys_out (host, may be NULL) receives at most cap key ids in
 * ascending order; *nkeys_out the full count; *is_large_out 1 for a large-key unit. */
int     kv_plan_unit(const kv_plan* plan, int unit, int* is_large_out, int* nkeys_out, int* keys_out, int cap);
/* Unit and arena element offset of a key. */
int     kv_plan_key(const kv_plan* plan, int key, int* unit_out, int64_t* arena_offset_out);
int64_t kv_plan_arena_numel(const kv_plan* plan);              /* fp32 elements incl. padding */

/* ------------------------------------------------------------------ chain (host only)
 * The launch-order state machine the store runs on every push, exposed so that the
 * ordering invariant can be checked without a GPU.  kv_chain_mark records the push
 * of one key (KV_ERR_STATE if the key is already marked and its unit has not run);
 * kv_chain_next_run then yields, repeatedly, maximal runs [first, first + n) of
 * consecutive ready units in ascending index, wrapping to unit 0 for the next
 * iteration; it returns 1 while it yields a run and 0 when nothing is ready.
 * A unit is ready when all its keys are marked; a ready unit still waits for every
 * lower unit of the same iteration (the paper's chain of write dependencies).
 * kv_chain_set_descending(1) reverses the order (last unit first, every unit waits for the
 * higher ones); a run is still reported by its lowest unit and its length.  Allowed only
 * between iterations (KV_ERR_STATE otherwise).
 */
int     kv_chain_create(kv_chain** out, const kv_plan* plan /* must outlive the chain */);
void    kv_chain_destroy(kv_chain* chain);
int     kv_chain_set_descending(kv_chain* chain, int descending);
int     kv_chain_mark(kv_chain* chain, int key);
int     kv_chain_next_run(kv_chain* chain, int* first_unit_out, int* n_units_out);
int     kv_chain_pending_keys(const kv_chain* chain);          /* marked, unit not yet run */
int     kv_chain_next_unit(const kv_chain* chain);             /* 0 when an iteration is complete */

/* ------------------------------------------------------------------ store
 * kv_init: KVStore.init for all keys at once (keys are 0..num_keys-1 in the linear
 * order of the tensors, as the paper assigns them).  Builds the plan, allocates the
 * fp32 weight and momentum arenas (zero-filled) on the current device and uploads
 * the tile tables.  hip_stream is a hipStream_t (NULL = the default stream) that
 * must outlive the store.  W in 1..KV_MAX_W.  flags: kv_flags.  tuning may be NULL.
 */
int kv_init(kv_store** out, int num_keys, const int64_t* key_numel /* host */, int grad_dtype, int W,
            size_t bucket_bytes, const kv_sgd_params* params /* host */, unsigned flags,
            const kv_tuning* tuning /* host or NULL */, void* hip_stream);
void kv_destroy(kv_store* store);                              /* drains the stream first; NULL is a no-op */

/* Initial value of a key (the paper broadcasts rank 0's value; here there is one
 * copy) and momentum restore.  src: numel fp32 values, device or host memory;
 * copied on the store's stream (the one given to kv_init, under every schedule), in order with
 * pushes and pulls of the key; src may be reused as soon as that stream's order allows. */
int kv_set_weights (kv_store* store, int key, const void* src_f32);
int kv_set_momentum(kv_store* store, int key, const void* src_f32);
/* Learning rate from the next launch on.  The paper's Evaluation section starts from 0.1 and grows the rate with
 * the mini-batch, i.e. with the number of GPUs, up to 1.0 at 256 GPUs; a schedule is a sequence of these calls. */
int kv_set_lr(kv_store* store, float lr);
/* All optimizer parameters at once (same rules as at kv_init; they take effect at the next launch),
 * and the ones in force; params_out->rescale is the resolved factor (1/W if it was given as <= 0). */
int kv_set_sgd_params(kv_store* store, const kv_sgd_params* params /* host */);
int kv_get_sgd_params(const kv_store* store, kv_sgd_params* params_out /* host */);

/*
 * kv_push: hands over the W gradient copies of one key (KVStore API section: a
 * push sums every gradient that carries the same key).  dev_grads: host array of W
 * device pointers, each to numel elements of the gradient dtype, aligned at least
 * to the element size (all W aligned to one vector of the launch shape -- at most 16 bytes for
 * fp32, 8 bytes for fp16 -- selects the vector path; buffers that start on a 128-byte cache line,
 * as separately allocated arrays do, are read fastest, see kv_wide_launches).
 * The gradients are read in place, asynchronously: they must stay valid and
 * unmodified until kv_wait returns or the stream is synchronised.  Never blocks.
 * When the push completes the next unit in order, that unit and every directly
 * following ready unit are launched as ONE kernel launch.
 */
int kv_push(kv_store* store, int key, const void* const* dev_grads /* host [W] */);
/* List form (the paper's push takes lists of keys and tensors): marks all keys
 * first, then launches; pushing all keys gives one launch per iteration.
 * dev_grads is a host array [nkeys * W], key-major.  Either every key of the list
 * is accepted or none is. */
int kv_push_list(kv_store* store, int nkeys, const int* keys /* host */, const void* const* dev_grads /* host */);
/*
 * Graph capture.  kv_push, kv_push_list and the pull functions may be called while the store's
 * stream is being captured into a HIP graph (chained schedule only); every replay of the graph then
 * repeats the launches with the gradient buffers and the optimizer parameters of the capture (the
 * replica table of kv_set_broadcast is read as it is at replay time).
 * Nothing can be uploaded during a capture, so the gradient buffers of every captured push must
 * have been pushed once before it (their pointers then sit in a cached device table); a capture
 * holds whole iterations.  A push that does not meet this returns KV_ERR_STATE and changes nothing.
 * The table a captured launch reads is kept until kv_release_captures or kv_destroy; at most 7
 * different sets of gradient buffers can be held this way (KV_ERR_STATE beyond).  Call
 * kv_release_captures once the graphs are gone; replaying one afterwards is undefined.
 * Every other call (kv_wait, kv_barrier, kv_set_*, timing) belongs outside the capture.  The launch
 * log and the launch counter count a captured launch once, when it is recorded.
 */
int kv_release_captures(kv_store* store);
/*
 * kv_push_list_noalloc: kv_push_list for callers that cannot allocate or upload: code under HIP graph
 * capture that pushes buffers the store has not seen before, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same values, same launch order.  The call allocates nothing on the host or
 * the device and copies nothing from host memory: the gradient-pointer table its launches read is a
 * file-scope device array that the library's code object carries (512 KiB on every GPU the library
 * runs on, held until the process ends), filled by a small kernel that takes the pointers in its
 * arguments (one fill launch per 384 pointers before each fused launch).
 *   - Limit: num_keys * W <= 65536 pointers; a larger store gets KV_ERR_ARG and nothing happens.
 *   - Chained schedule only (KV_ERR_STATE otherwise).
 *   - Every store on a GPU shares that GPU's array, which keeps the rows of the last call.  Calls on one
 *     stream are ordered by the stream.  Calls whose launches can overlap on one GPU (stores on different
 *     streams, or graph replays racing with eager calls on another stream) race on the rows they share:
 *     the caller must order them.
 *   - May be called while the stream is captured; the capture needs no earlier push of the same buffers
 *     and pins no table.  A replay rewrites the rows it needs before it reads them.
 */
int kv_push_list_noalloc(kv_store* store, int nkeys, const int* keys /* host */, const void* const* dev_grads /* host */);
/* The launch tuning in force (the defaults resolved, or what KV_FLAG_AUTOTUNE has chosen so far);
 * *tuning_done_out (may be NULL) is 0 while a store that tunes itself is still trying shapes. */
int kv_get_tuning(const kv_store* store, kv_tuning* tuning_out /* host */, int* tuning_done_out /* host */);
/* Gradient buffers off the cache-line grid: a store whose default shape is one element per lane, or two with 8 and
 * more ranks (that is: 8 and more fp32 ranks; 8, 16, or 24 and more fp16 ranks; not when kv_tuning fixes lane_elems
 * or unroll, nor while KV_FLAG_AUTOTUNE is trying shapes) launches with four elements per lane instead when more than half of a launch's gradient elements lie in
 * keys with a gradient pointer that is not a multiple of 128 bytes (views into a flat buffer) while all of them are
 * multiples of one 4-element vector.  Same bits, fewer cache lines fetched twice.  *count_out = launches so far that
 * took that shape (kv_get_tuning keeps reporting the default one). */
int kv_wide_launches(const kv_store* store, int64_t* count_out);

/*
 * kv_pull: copies the key's current weights (numel fp32) to dev_out on the store's
 * stream; after a push of the same key it observes the updated value (if the key's
 * unit has not been launched yet the copy is queued and issued right after that
 * launch).  kv_pull_grad copies the raw fp32 sum s of the last step (the value the
 * paper's pull returns); it needs KV_FLAG_KEEP_SUM, else KV_ERR_STATE.
 */
int kv_pull(kv_store* store, int key, void* dev_out_f32);
int kv_pull_grad(kv_store* store, int key, void* dev_out_f32);
int kv_pull_momentum(kv_store* store, int key, void* dev_out_f32);
/* List form of kv_pull (the paper's pull takes lists of keys and tensors): dev_out_f32 is a host
 * array of nkeys device pointers, 4-byte aligned (16-byte alignment keeps the 128-bit path).  Keys
 * that are not waiting for a launch are gathered by one kernel per run of keys that are neighbours
 * in the arena (all keys: one launch); otherwise, and whenever the stream is being captured into a graph
 * (the gather's destination table is uploaded from reusable staging memory, which a replay must not
 * read again), the list is served key by key as kv_pull would. */
int kv_pull_list(kv_store* store, int nkeys, const int* keys /* host */, void* const* dev_out_f32 /* host */);
/* Zero-copy pull: device address of the key's weights inside the arena (numel fp32,
 * 256-byte aligned, valid until kv_destroy; contents change with every step). */
int kv_weights_ptr(kv_store* store, int key, void** dev_ptr_out);

/*
 * kv_set_broadcast: the third phase of the paper's collective (every GPU receives the final
 * result; its pull does this by copying the aggregate back into every worker's tensor), fused
 * into the update: from the next launch on, the kernel that computes the key's new
 * weights also writes them to n_replicas caller-owned device buffers of numel elements each, as
 * fp32 (dtype KV_F32) or rounded to nearest-even fp16 (KV_F16).  dev_dst: host array of n_replicas
 * device pointers, aligned to the element (all of them aligned to 16 bytes for fp32 replicas, 8 bytes
 * for fp16 replicas, keeps the vector path).
 * Every key of a store must use the same n_replicas and dtype (KV_ERR_STATE otherwise); n_replicas = 0
 * removes the key's replicas.  Blocks until the store's streams are idle.  The replicas must stay
 * valid while pushes of the key can still launch.
 */
int kv_set_broadcast(kv_store* store, int key, int n_replicas, void* const* dev_dst /* host [n_replicas] */, int dtype);
/* The paper's KVStore.init ends with a broadcast of the initial value to every worker: copies the CURRENT
 * weights of `key` (-1: of every key) to the replicas registered with kv_set_broadcast, in the
 * replicas' dtype, on the key's stream and in order with its pushes and kv_set_weights.  Keys
 * without replicas are skipped; KV_ERR_STATE if the key is pushed and waits for its launch. */
int kv_broadcast_weights(kv_store* store, int key);

/* Makes the store's stream wait (on the GPU, not the host) for hip_event (a hipEvent_t recorded on
 * another stream): the read dependency of later pushes on gradients that the other stream produces. */
int kv_wait_event(kv_store* store, void* hip_event);

/*
 * kv_wait(key >= 0): blocks the host until the key's last launched update and every pull of the key issued
 * after it are complete (the paper's WaitToRead on one tensor); KV_ERR_INCOMPLETE, without blocking, if the key is
 * pushed but its unit cannot be launched yet.  Work on other streams of the concurrent schedule never delays the
 * return; work queued later on the key's own stream delays it by a bounded amount: an event record per launch
 * costs about as much host time as the launch itself, so a stream records a completion event only after every
 * 8th launch (or pull) that may be waited for, or earlier once 64 MB of launch traffic have gone out since its
 * last one, into a ring of 256, and the wait is for the first event of the key's stream at or after the key's
 * launch: at most 7 later launches, or 64 MB of later traffic, whichever is less.  When the stream has recorded
 * none since (or the ring has moved on), the wait is for the stream as it stands; so it is after a launch that
 * covered every unit of the store (one launch per iteration: nothing is recorded on that path, and the stream
 * holds nothing else of the iteration).
 * kv_wait(-1): barrier (the paper's Kvstore.barrier): drains the stream, then
 * returns KV_ERR_INCOMPLETE if an iteration is only partly pushed or launched.
 */
int kv_wait(kv_store* store, int key);

/*
 * kv_set_schedule: the paper's KVStore.create("type").  Allowed only between iterations
 * (KV_ERR_STATE while pushed keys wait); drains all streams first.  n_streams (1..KV_MAX_STREAMS)
 * and outstanding (>= 0) are read for KV_SCHED_CONCURRENT only; the extra streams are created by
 * the store at default priority.  In the concurrent schedule a key's launch and its pulls run on
 * the key's stream, ordered after everything issued earlier on the stream given to kv_init (so
 * gradients and pull destinations must stay valid until kv_wait(key) or kv_barrier); work the caller issues afterwards on that stream is ordered after a key only through
 * kv_wait(key) or kv_barrier.  In the launch log per-key launches appear as (key, 0).
 * kv_barrier: the paper's Kvstore.barrier: blocks until nothing launched so far is outstanding
 * on any stream.  Unlike kv_wait(-1) it does not report an incomplete iteration.
 */
int kv_set_schedule(kv_store* store, int schedule, int n_streams, int outstanding);
int kv_barrier(kv_store* store);

/* ------------------------------------------------------------------ introspection
 * The plan in use (owned by the store). */
const kv_plan* kv_store_plan(const kv_store* store);
/* Launch log: total number of kernel launches so far in *total_out; the most
 * recent min(total, cap) launches, oldest first, as (lowest unit, n_units) pairs. */
int kv_launch_log(const kv_store* store, int64_t* total_out, int* first_unit_out, int* n_units_out, int cap);
/* GPU time between two points of the store's stream, measured with HIP events:
 * begin records an event; end records another, waits for it and returns the
 * elapsed milliseconds and the number of kernel launches issued in between. */
int kv_timing_begin(kv_store* store);
int kv_timing_end(kv_store* store, float* ms_out, int64_t* launches_out);
/* Between begin and end, kv_timing_mark records one more event on the store's stream (at most
 * KV_MAX_TIMING_MARKS of them; it does not wait).  After kv_timing_end, kv_timing_intervals writes
 * the milliseconds from begin to the first mark and between consecutive marks into ms_out (host,
 * at most cap values) and returns how many it wrote: per-step times without a host wait per step. */
int kv_timing_mark(kv_store* store);
int kv_timing_intervals(kv_store* store, float* ms_out, int cap);
/* Message for the last failure on this store (or, with NULL, of the last failed
 * kv_init / kv_plan_create / kv_chain_create on this thread).  Never NULL. */
const char* kv_last_error(const kv_store* store);

#ifdef __cplusplus
}
#endif
#endif /* KV_H */
