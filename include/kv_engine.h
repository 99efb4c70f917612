/*
 * kv_engine.h - C ABI of a minimal dependency engine (host side).
 *
 * It follows the paper's "Dependency Tracking" and "Task Execution" sections: every
 * operation is pushed by one thread together with the tags (variables) it only reads
 * and the tags it mutates, e.g. b = a + 1 is push(fn, read = {a}, mutate = {b}).  The
 * engine keeps one queue of pending operations per variable and one counter of unmet
 * dependencies per operation; an operation whose counter reaches zero is handed to a
 * pool of worker threads.  Back-to-back reads of a variable are released together and
 * may run concurrently; writes to a variable run one at a time, in the order they were
 * pushed, and never while a read of it runs.  The paper uses exactly that last property
 * to chain its collectives: every aggregation mutates one extra "dummy" variable.
 *
 * Operations are plain C callbacks, void fn(void* arg).  The engine never touches the
 * GPU itself; the ready-made callbacks at the end of this header do.
 *
 * All functions return KV_OK (0) or a negative kv_status (see kv.h).  Only one thread
 * may call kv_engine_new_var and kv_engine_push (as in the paper, where only the main
 * thread issues operations); the wait functions may be called from that thread only.
 */
#ifndef KV_ENGINE_H
#define KV_ENGINE_H

#include <stddef.h>
#include <stdint.h>

#include "kv.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kv_engine kv_engine;          /* opaque */
typedef void (*kv_engine_fn)(void* arg);

/* n_threads worker threads, 1..256.  The engine is freed by kv_engine_destroy, which first
 * waits for everything pushed so far. */
int  kv_engine_create(kv_engine** out, int n_threads);
void kv_engine_destroy(kv_engine* engine);

/* A new variable (tag); ids count up from 0. */
int  kv_engine_new_var(kv_engine* engine, int* var_out);

/*
 * Pushes one operation.  read_vars / mutate_vars: host arrays of variable ids (may be NULL
 * when the count is 0); a variable listed in both, or twice, counts once (as mutated if it
 * is mutated).  arg must stay valid until the operation has run.  Never blocks on the
 * operation; returns KV_ERR_KEY for an unknown variable id.
 */
int  kv_engine_push(kv_engine* engine, kv_engine_fn fn, void* arg, const int* read_vars, int n_read,
                    const int* mutate_vars, int n_mutate);

/* Blocks until every operation pushed so far that reads or mutates `var` has run (the
 * paper's WaitToRead waits for the writes only; this waits for the reads too). */
int  kv_engine_wait_var(kv_engine* engine, int var);
/* Blocks until everything pushed so far has run. */
int  kv_engine_wait_all(kv_engine* engine);

/* Counters since creation: operations run, and the largest number that ran at the same time. */
int  kv_engine_stats(const kv_engine* engine, int64_t* ops_run_out, int* max_concurrent_out);

/* ------------------------------------------------------------------ ready-made operations
 * Callbacks for kv_engine_push whose arg is the struct shown; each stores its kv_status in
 * `status`.  They let a training loop be expressed as in the paper's listings: a producer
 * operation mutates the gradient's variable, the push operation reads it and mutates the
 * store's variable (the "dummy" that serialises all calls into the store, which is not
 * thread-safe).
 */

/* Stand-in for a backward operator that produces a gradient: on hip_stream every lane first
 * runs `spin` (>= 0) dependent multiply-adds (compute without memory traffic), then `bytes`
 * bytes (multiple of 16, both pointers 16-byte aligned) are copied from src to dst, then
 * record_event (may be NULL) is recorded on that stream.  max_workgroups caps the kernel's grid
 * (workgroups of 256 lanes; 0 = as many as the copy needs, at most 2048, which fills every compute
 * unit): 256 or 512 leave most wave slots of the chip to whatever else is running. */
typedef struct kv_op_copy_args {
    void*       dev_dst;
    const void* dev_src;
    size_t      bytes;
    void*       hip_stream;
    void*       record_event;   /* hipEvent_t or NULL */
    int         spin;
    int         status;
    int         max_workgroups;
} kv_op_copy_args;
void kv_op_copy(void* arg /* kv_op_copy_args* */);

/* KVStore push of one key: makes the store's stream wait for wait_events[0..n_events)
 * (hipEvent_t; the read dependency on the gradients, which another stream produces), then
 * calls kv_push(store, key, dev_grads). */
typedef struct kv_op_push_args {
    kv_store*          store;
    int                key;
    const void* const* dev_grads;      /* host array [W], valid until the operation has run */
    void* const*       wait_events;    /* host array [n_events] or NULL */
    int                n_events;
    int                status;
} kv_op_push_args;
void kv_op_push(void* arg /* kv_op_push_args* */);

/* HIP events for the two operations above (timing disabled); thin wrappers so that a caller
 * without a HIP binding can create them. */
int  kv_event_create(void** event_out);
void kv_event_destroy(void* event);

#ifdef __cplusplus
}
#endif
#endif /* KV_ENGINE_H */
