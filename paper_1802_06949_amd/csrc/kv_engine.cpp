// Minimal dependency engine (see include/kv_engine.h).
//
// Per variable: a queue of operations that still wait for it, the number of reads
// of it that are running and whether a write of it is running.  Per operation: a
// counter of dependencies not yet granted (the paper's atomic counter).  A read is
// granted when no write runs or waits ahead of it; consecutive queued reads are
// granted together; a write is granted when nothing runs on the variable and it is
// at the head of the queue, so writes run one at a time in push order.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <deque>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

#include "../../include/kv_engine.h"
#include "kv_kernels.hpp"

namespace {

struct Op {
    kv_engine_fn fn = nullptr;
    void* arg = nullptr;
    std::atomic<int> pending{0};
    std::vector<int> reads, writes;
};

struct Waiting {
    Op* op;
    bool write;
};

struct Var {
    std::deque<Waiting> queue;
    int running_reads = 0;
    bool running_write = false;
    int64_t outstanding = 0;      // operations pushed on this variable and not yet finished
};

}  // namespace

struct kv_engine {
    std::mutex mu;
    std::condition_variable ready_cv;   // workers: something to run, or shutting down
    std::condition_variable done_cv;    // waiters: an operation finished
    std::deque<Op*> ready;
    std::vector<Var> vars;
    std::vector<std::thread> workers;
    int64_t outstanding = 0;
    int64_t ops_run = 0;
    int running = 0;
    int max_running = 0;
    bool stop = false;

    // callers hold mu
    void grant(Op* op) {
        if (op->pending.fetch_sub(1) == 1) {
            ready.push_back(op);
            ready_cv.notify_one();
        }
    }

    void release(Var& v) {
        while (!v.queue.empty()) {
            Waiting head = v.queue.front();
            if (head.write) {
                if (v.running_reads == 0 && !v.running_write) {
                    v.running_write = true;
                    v.queue.pop_front();
                    grant(head.op);
                }
                return;
            }
            if (v.running_write) return;
            ++v.running_reads;              // a run of queued reads goes out together
            v.queue.pop_front();
            grant(head.op);
        }
    }

    void worker() {
        std::unique_lock<std::mutex> lk(mu);
        for (;;) {
            ready_cv.wait(lk, [&] { return stop || !ready.empty(); });
            if (ready.empty()) return;      // stop requested and nothing left
            Op* op = ready.front();
            ready.pop_front();
            ++running;
            max_running = std::max(max_running, running);
            lk.unlock();
            op->fn(op->arg);
            lk.lock();
            --running;
            ++ops_run;
            for (int r : op->reads) {
                Var& v = vars[(size_t)r];
                if (--v.running_reads == 0) release(v);
                --v.outstanding;
            }
            for (int w : op->writes) {
                Var& v = vars[(size_t)w];
                v.running_write = false;
                release(v);
                --v.outstanding;
            }
            --outstanding;
            delete op;
            done_cv.notify_all();
        }
    }
};

extern "C" {

int kv_engine_create(kv_engine** out, int n_threads) {
    if (!out || n_threads < 1 || n_threads > 256) return KV_ERR_ARG;
    *out = nullptr;
    kv_engine* e = new (std::nothrow) kv_engine();
    if (!e) return KV_ERR_NOMEM;
    try {
        for (int i = 0; i < n_threads; ++i) e->workers.emplace_back([e] { e->worker(); });
    } catch (...) {
        kv_engine_destroy(e);
        return KV_ERR_NOMEM;
    }
    *out = e;
    return KV_OK;
}

void kv_engine_destroy(kv_engine* engine) {
    if (!engine) return;
    {
        std::unique_lock<std::mutex> lk(engine->mu);
        engine->done_cv.wait(lk, [&] { return engine->outstanding == 0; });
        engine->stop = true;
    }
    engine->ready_cv.notify_all();
    for (auto& t : engine->workers)
        if (t.joinable()) t.join();
    delete engine;
}

int kv_engine_new_var(kv_engine* engine, int* var_out) {
    if (!engine || !var_out) return KV_ERR_ARG;
    std::lock_guard<std::mutex> lk(engine->mu);
    try {
        engine->vars.emplace_back();
    } catch (const std::bad_alloc&) {
        return KV_ERR_NOMEM;
    }
    *var_out = (int)engine->vars.size() - 1;
    return KV_OK;
}

int kv_engine_push(kv_engine* engine, kv_engine_fn fn, void* arg, const int* read_vars, int n_read,
                   const int* mutate_vars, int n_mutate) {
    if (!engine || !fn || n_read < 0 || n_mutate < 0 || (n_read > 0 && !read_vars) || (n_mutate > 0 && !mutate_vars))
        return KV_ERR_ARG;
    Op* op = new (std::nothrow) Op();
    if (!op) return KV_ERR_NOMEM;
    std::lock_guard<std::mutex> lk(engine->mu);
    const int nv = (int)engine->vars.size();
    try {
        op->writes.assign(mutate_vars, mutate_vars + n_mutate);
        std::sort(op->writes.begin(), op->writes.end());
        op->writes.erase(std::unique(op->writes.begin(), op->writes.end()), op->writes.end());
        for (int i = 0; i < n_read; ++i)
            if (!std::binary_search(op->writes.begin(), op->writes.end(), read_vars[i])) op->reads.push_back(read_vars[i]);
        std::sort(op->reads.begin(), op->reads.end());
        op->reads.erase(std::unique(op->reads.begin(), op->reads.end()), op->reads.end());
    } catch (const std::bad_alloc&) {
        delete op;
        return KV_ERR_NOMEM;
    }
    for (int v : op->reads)
        if (v < 0 || v >= nv) { delete op; return KV_ERR_KEY; }
    for (int v : op->writes)
        if (v < 0 || v >= nv) { delete op; return KV_ERR_KEY; }
    op->fn = fn;
    op->arg = arg;
    op->pending.store(1);                    // held until every dependency is registered
    for (int r : op->reads) {
        Var& v = engine->vars[(size_t)r];
        ++v.outstanding;
        if (!v.running_write && v.queue.empty()) {
            ++v.running_reads;
        } else {
            op->pending.fetch_add(1);
            v.queue.push_back(Waiting{op, false});
        }
    }
    for (int w : op->writes) {
        Var& v = engine->vars[(size_t)w];
        ++v.outstanding;
        if (!v.running_write && v.running_reads == 0 && v.queue.empty()) {
            v.running_write = true;
        } else {
            op->pending.fetch_add(1);
            v.queue.push_back(Waiting{op, true});
        }
    }
    ++engine->outstanding;
    engine->grant(op);
    return KV_OK;
}

int kv_engine_wait_var(kv_engine* engine, int var) {
    if (!engine) return KV_ERR_ARG;
    std::unique_lock<std::mutex> lk(engine->mu);
    if (var < 0 || var >= (int)engine->vars.size()) return KV_ERR_KEY;
    engine->done_cv.wait(lk, [&] { return engine->vars[(size_t)var].outstanding == 0; });
    return KV_OK;
}

int kv_engine_wait_all(kv_engine* engine) {
    if (!engine) return KV_ERR_ARG;
    std::unique_lock<std::mutex> lk(engine->mu);
    engine->done_cv.wait(lk, [&] { return engine->outstanding == 0; });
    return KV_OK;
}

int kv_engine_stats(const kv_engine* engine, int64_t* ops_run_out, int* max_concurrent_out) {
    if (!engine) return KV_ERR_ARG;
    kv_engine* e = const_cast<kv_engine*>(engine);
    std::lock_guard<std::mutex> lk(e->mu);
    if (ops_run_out) *ops_run_out = e->ops_run;
    if (max_concurrent_out) *max_concurrent_out = e->max_running;
    return KV_OK;
}

// ------------------------------------------------------------------ ready-made operations
void kv_op_copy(void* arg) {
    kv_op_copy_args* a = static_cast<kv_op_copy_args*>(arg);
    if (!a) return;
    if (!a->dev_dst || !a->dev_src || (a->bytes & 15u) || ((uintptr_t)a->dev_dst & 15u) || ((uintptr_t)a->dev_src & 15u) ||
        a->spin < 0 || a->max_workgroups < 0) {
        a->status = KV_ERR_ARG;
        return;
    }
    a->status = kv_launch_busy_copy(a->dev_dst, a->dev_src, a->bytes, a->spin, a->max_workgroups, static_cast<hipStream_t>(a->hip_stream)) ==
                        hipSuccess
                    ? KV_OK
                    : KV_ERR_HIP;
    if (a->status == KV_OK && a->record_event) {
        if (hipEventRecord(static_cast<hipEvent_t>(a->record_event), static_cast<hipStream_t>(a->hip_stream)) != hipSuccess)
            a->status = KV_ERR_HIP;
    }
}

void kv_op_push(void* arg) {
    kv_op_push_args* a = static_cast<kv_op_push_args*>(arg);
    if (!a) return;
    a->status = KV_OK;
    for (int i = 0; i < a->n_events && a->status == KV_OK; ++i)
        if (a->wait_events && a->wait_events[i]) a->status = kv_wait_event(a->store, a->wait_events[i]);
    if (a->status == KV_OK) a->status = kv_push(a->store, a->key, a->dev_grads);
}

int kv_event_create(void** event_out) {
    if (!event_out) return KV_ERR_ARG;
    hipEvent_t ev = nullptr;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) return KV_ERR_HIP;
    *event_out = ev;
    return KV_OK;
}

void kv_event_destroy(void* event) {
    if (event) (void)hipEventDestroy(static_cast<hipEvent_t>(event));
}

}  // extern "C"
