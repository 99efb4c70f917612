/*
 * kv_diag.h - measurement helpers of the MI355X key-value aggregation library.
 *
 * Nothing here is part of the method (include/kv.h is): these are plain kernels of known size
 * against which hardware byte counters are calibrated, measured ceilings of the memory system that
 * the fused kernel's rate is put next to, a cache flush for cold-state timing and an empty launch
 * for the latency floor of launch-bound workloads.  Same library, same conventions: KV_OK or a
 * negative kv_status; kv_last_error(NULL) gives the message; pointers are device memory unless
 * marked host; hip_stream is a hipStream_t (NULL = the default stream); nothing is allocated.
 */
#ifndef KV_DIAG_H
#define KV_DIAG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Plain streaming copy kernel (float4 grid-stride) of `bytes` bytes (multiple of 16,
 * both pointers 16-byte aligned) on hip_stream: the known-size kernel against which
 * hardware byte counters are calibrated. */
int kv_copy_bytes(void* dev_dst, const void* dev_src, size_t bytes, void* hip_stream);
/* Plain streaming read kernel: reads `bytes` bytes (multiple of 16, pointer 16-byte aligned) and
 * writes nothing.  With kv_copy_bytes it gives the measured read and copy ceilings of the GPU that the
 * fused kernel's rate is put next to. */
int kv_read_bytes(const void* dev_src, size_t bytes, void* hip_stream);
/* Measured ceiling for a MIX of streams with 16 bytes per lane and stream (one workgroup per 4 KB
 * of every stream, all loads in flight before the first store): every lane sums its 16-byte
 * vector of n_read buffers (1, 2, 4, 8, 16 or 32) and stores the sum to each of n_write buffers
 * (0..8).  dev_bufs: host array of n_read + n_write device pointers, read buffers first, each to
 * `bytes` bytes (multiple of 16), 16-byte aligned, none overlapping a written one.  KV_ERR_ARG otherwise. */
int kv_stream_mix(void* const* dev_bufs /* host */, int n_read, int n_write, size_t bytes, void* hip_stream);

/* Cache flush for cold-state timing: a pass of plain (cached, not non-temporal) accesses over `bytes` bytes
 * (multiple of 16, pointer 16-byte aligned).  Run over a buffer of at least twice the 256 MiB memory-side cache
 * it leaves nothing else resident in L2 or in that cache: the state in which a training iteration finds the
 * weights after a forward and backward pass.  dirty = 0: loads only, the buffer's lines are left clean;
 * dirty = 1: read-modify-write (adds 1 to the first float of every vector), the lines are left modified and
 * have to be written back when the next kernel displaces them. */
int kv_evict_caches(void* dev_buf, size_t bytes, int dirty, void* hip_stream);
/* Launches `count` (>= 1) empty kernels (one workgroup each) back to back on hip_stream, from native code: timed
 * with events around the call, the floor under any launch-bound step. */
int kv_null_launch(int count, void* hip_stream);

/* kv_push_list(store, nkeys, keys, dev_grads) `reps` (>= 1) times back to back from native code, the same buffers
 * every time: the rate at which a native caller can step a launch-bound store, with no interpreter between the
 * launches (a store of a few hundred KB per step is otherwise timed by its binding).  Stops at the first call that
 * fails and returns its status. */
struct kv_store;
int kv_push_list_repeat(struct kv_store* store, int nkeys, const int* keys /* host */,
                        const void* const* dev_grads /* host */, int reps);

/* Completion events recorded so far for kv_wait(key) (see there: one per 8 launches of a stream, or per 64 MB of
 * launch traffic): what a test reads to see that a run of small launches shares events and a large one gets its own. */
int kv_completion_events(const struct kv_store* store, int64_t* count_out /* host */);

#ifdef __cplusplus
}
#endif
#endif /* KV_DIAG_H */
