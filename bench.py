#!/usr/bin/env python3
"""Benchmark of the fused W-way gradient reduction + SGD update on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic gradients:
one list push of every key (host scheduling, pointer-table lookup, one fused
kernel launch covering all units), with the updated weights available in place
(zero-copy pull) and a barrier after the last timed step.  Inputs are resident in
HBM before the timed region starts.

Prints ONE JSON line.  `value` is aggregated gradient bytes per second
(N * W * sizeof(grad) / t_step); `roofline` prices the fused kernel's algorithmic
bytes (N * (W * sizeof(grad) + 16) per launch) against the 8 TB/s HBM peak, with
the launch duration measured by HIP events on the store's stream;
`cpu_baseline` is the CPU oracle timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
METRIC = "aggregated gradient bytes/s (GB/s, % HBM peak) for W-way reduce+SGD update"


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (default 6000; 30 with --overlap)")
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--config", type=int, default=3, help="benchmark configuration 1..5 (3 = ResNet-50-shaped, W=8)")
    ap.add_argument("--ranks", type=int, default=0, help="override the configuration's W (characterisation runs)")
    ap.add_argument("--grad-dtype", choices=["f32", "f16"], default=None, help="override the gradient dtype")
    ap.add_argument("--sets", type=int, default=2, help="distinct gradient sets cycled through (fresh buffers each step)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cold-steps", type=int, default=40,
                    help="steps of the cold-state legs: before each one a plain pass over 1 GiB of unrelated memory "
                         "flushes L2 and the memory-side cache, outside the step's event pair (0 = skip)")
    ap.add_argument("--cold-evict", choices=["both", "clean", "dirty"], default="both",
                    help="which cold-state legs run (profiling runs that want one kind of launch in the trace)")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the legs on the other benchmark configurations (1, 2, 4, 5 and 6)")
    ap.add_argument("--cpu-seconds", type=float, default=8.0,
                    help="CPU work per oracle leg (single thread, all cores); whole steps are run until it is used up")
    ap.add_argument("--calib-copy", type=int, default=0, metavar="N",
                    help="also launch the plain copy kernel N times on 1 GiB (byte-counter calibration)")
    ap.add_argument("--ceilings", action="store_true", help="also measure the plain copy kernel on 1 GiB (context)")
    ap.add_argument("--ceilings-data", choices=["random", "zeros"], default="random",
                    help="--ceilings: contents of the buffers (on this GPU all-zero buffers move measurably faster "
                         "than random data; the benchmark's gradients and weights are random)")
    ap.add_argument("--pull-copy", action="store_true", help="also time a copying pull of every key (reported apart)")
    ap.add_argument("--schedule", choices=["chained", "funnel", "concurrent"], default="chained",
                    help="chained = one merged launch per step (headline); funnel / concurrent = one launch per key")
    ap.add_argument("--push-mode", choices=["list", "each"], default="list",
                    help="list = one kv_push_list per step (headline); each = one kv_push per key, in key order")
    ap.add_argument("--lazy", action="store_true", help="KV_FLAG_LAZY_LAUNCH: single pushes merge into one launch")
    ap.add_argument("--streams", type=int, default=4, help="concurrent schedule: number of streams")
    ap.add_argument("--outstanding", type=int, default=0, help="concurrent schedule: barrier after this many keys")
    ap.add_argument("--broadcast", choices=["none", "f32", "f16"], default="none",
                    help="also write the new weights to --replicas replica buffers per key in the same kernel")
    ap.add_argument("--replicas", type=int, default=0, help="replica buffers per key (default: W)")
    ap.add_argument("--overlap", action="store_true",
                    help="instead of the headline: engine-driven loop with synthetic backward operators on a second "
                         "stream, reported as backward only / aggregation only / serial / overlapped")
    ap.add_argument("--spin", type=int, default=20000, help="--overlap: multiply-adds per lane of the largest producer")
    ap.add_argument("--engine-threads", type=int, default=2)
    ap.add_argument("--producer-workgroups", type=int, default=0,
                    help="--overlap: cap of every producer's grid (0 = up to 2048 workgroups, which fill the chip; 256 = "
                         "one workgroup of 256 lanes per compute unit)")
    ap.add_argument("--producer-bytes", type=int, default=0,
                    help="--overlap: a producer copies only this many leading bytes of its gradient (0 = all of it), so that "
                         "it spends its time computing")
    ap.add_argument("--flat-grads", action="store_true",
                    help="each rank's gradients of all keys live in ONE buffer (keys at 256-byte aligned offsets) "
                         "instead of one allocation per key and rank")
    ap.add_argument("--rank-skew", type=int, default=0,
                    help="--flat-grads: rank r's buffer starts r * this many bytes into its allocation (multiple of 16)")
    ap.add_argument("--view-offset", type=int, default=0,
                    help="--flat-grads: every rank's views start this many bytes into its allocation (multiple of 16): "
                         "32 puts every gradient buffer off the 128-byte line grid")
    ap.add_argument("--graph", action="store_true",
                    help="record one iteration per gradient set into a HIP graph (on a side stream, after eager "
                         "warm-up steps) and time replays of the graphs instead of direct launches")
    ap.add_argument("--autotune", action="store_true",
                    help="KV_FLAG_AUTOTUNE: the store tries launch shapes during (at least 45) warm-up steps and keeps "
                         "the fastest; the chosen tuning is reported in config.tuning")
    ap.add_argument("--keep-sum", action="store_true",
                    help="the kernel also stores the raw fp32 sums (what the paper's pull returns): +4 bytes per element")
    ap.add_argument("--unroll", type=int, default=0)
    ap.add_argument("--lane-elems", type=int, default=0)
    ap.add_argument("--resident-workgroups", type=int, default=0)
    ap.add_argument("--workgroups-per-cu", type=int, default=-1)
    ap.add_argument("--nontemporal", type=int, default=-1)
    ap.add_argument("--xcd-remap", type=int, default=-1)
    ap.add_argument("--run-time-w", action="store_true",
                    help="run the kernel that takes W at run time even where one built for this W exists")
    ap.add_argument("--gen-threads", type=int, default=min(16, os.cpu_count() or 1))
    return ap.parse_args()


def kernel_sources_sha256() -> str:
    """Fingerprint of everything the library is built from (csrc/ and the build script): ties a committed counter
    summary to the binary that is being timed."""
    import hashlib
    h = hashlib.sha256()
    pkg = os.path.join(ROOT, "paper_1802_06949_amd")
    files = [os.path.join(pkg, "build.py")] + sorted(os.path.join(pkg, "csrc", f) for f in os.listdir(os.path.join(pkg, "csrc")))
    for f in files:
        h.update(os.path.basename(f).encode() + b"\0")
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def read_traffic(workload: str):
    """HBM bytes per launch from the committed counter summary of this workload, and where it comes from."""
    name = f"hbm_traffic_{workload}.txt"
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None, None
    vals, meta = {}, {"file": f"profiles/{name}"}
    with open(path) as f:
        for line in f:
            body = line.lstrip("# ").strip()
            for tag in ("measured_at_commit", "measured_on", "kernel_sources_sha256"):
                if body.startswith(tag + ":"):
                    meta[tag] = body.split(":", 1)[1].strip()
            if ":" in line and not line.lstrip().startswith("#"):
                k, v = line.split(":", 1)
                try:
                    vals[k.strip()] = float(v.split()[0])
                except (ValueError, IndexError):
                    pass
    if "fetch_bytes_per_launch" in vals and "write_bytes_per_launch" in vals:
        meta["note"] = "rocprofv3 FETCH_SIZE / WRITE_SIZE between L2 and the fabric, from that earlier run, not from this one"
        if "kernel_sources_sha256" in meta:
            # was the library that run profiled built from the sources this run's library is built from?
            meta["library_sources_unchanged_since"] = meta.pop("kernel_sources_sha256") == kernel_sources_sha256()
        return vals["fetch_bytes_per_launch"] + vals["write_bytes_per_launch"], meta
    return None, None


MALL_BYTES = 256 << 20          # memory-side cache of the MI355X
EVICT_BYTES = 1 << 30


def device_gradients(cfg, nsets: int, seed: int):
    """Seeded gradients drawn on the GPU (timing legs of the other configurations: values do not change the time of a
    bandwidth-bound kernel, and 2.2e9 host draws for the VGG-16 shape would take longer than every timed leg)."""
    import torch
    import workloads as wl
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    sigma, zeros = wl.key_sigma(cfg), wl.zero_keys(cfg)
    tdt = torch.float32 if cfg.grad_dtype == "f32" else torch.float16
    sets = []
    for _ in range(nsets):
        one = []
        for k, n in enumerate(cfg.numel):
            if k in zeros:
                one.append([torch.zeros(n, dtype=tdt, device="cuda") for _ in range(cfg.W)])
            else:
                one.append([(torch.randn(n, device="cuda", generator=gen) * float(sigma[k])).to(tdt) for _ in range(cfg.W)])
        sets.append(one)
    return sets


def launch_floor_us(kv, reps: int = 2000) -> float:
    """Average time per launch of an empty kernel, back to back on the current stream."""
    import torch
    kv.null_launch(50)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    kv.null_launch(reps)                 # one native loop: no interpreter between the launches
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def cold_leg(kv, store, do_step, steps: int, evict_buf, dirty: bool, alg_bytes_step: float):
    """Steps that find nothing of theirs in L2 or the memory-side cache: a plain pass over 1 GiB of unrelated memory
    runs before each step, outside the step's pair of events (all on the store's stream)."""
    if steps <= 0:
        return None
    for i in range(2):
        kv.evict_caches(evict_buf, EVICT_BYTES, dirty)
        do_step(i)
    store.wait()
    before = store.launch_log(0)[0]
    store.timing_begin()
    for i in range(steps):
        kv.evict_caches(evict_buf, EVICT_BYTES, dirty)
        store.timing_mark()
        do_step(i)
        store.timing_mark()
    store.wait()
    store.timing_end()
    launches = store.launch_log(0)[0] - before
    iv = store.timing_intervals()[1::2]
    total_s = sum(iv) * 1e-3
    lps = launches / steps
    launch_s = total_s / max(launches, 1)
    achieved = alg_bytes_step / max(lps, 1e-9) / launch_s / 1e9
    srt = sorted(iv)
    return {
        "evict": "1 GiB plain read-modify-write pass before every step: caches full of modified unrelated lines, which the "
                 "step's own allocations force back to memory inside the timed launch (256 MiB of foreign write-back, about "
                 "as much as the step leaves modified itself: the steady state with all write-back on the clock)" if dirty else
                 "1 GiB plain read pass before every step: caches full of clean unrelated lines; the step's own w' and m' end "
                 "it modified in the memory-side cache and are written back after the timed launch (write-back deferred)",
        "achieved": round(achieved, 2),
        "frac": round(achieved / HBM_PEAK_GBPS, 4),
        "avg_launch_us": round(launch_s * 1e6, 3),
        "median_step_us": round(srt[len(srt) // 2] * 1e3, 3),
        "steps": steps,
    }


def other_config_leg(kv, cfg_id: int, evict_buf, cold_steps: int, floor_us: float):
    """One of the other benchmark configurations, in this process, same event method as the headline."""
    import torch
    import workloads as wl
    cfg = wl.get_config(cfg_id)
    K, N = len(cfg.keys), cfg.total_numel
    nsets = 1 if cfg.algorithmic_bytes_per_step > (4 << 30) else 2
    dev_sets = device_gradients(cfg, nsets, 1000 + cfg_id)
    store = kv.KVStore(cfg.numel, cfg.W, cfg.grad_dtype, cfg.bucket_bytes, lr=cfg.lr, momentum=cfg.momentum, wd=cfg.wd)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(2000 + cfg_id)
    for k, n in enumerate(cfg.numel):
        if n:
            store.set_weights(k, torch.randn(n, device="cuda", generator=gen) * 0.05)
    lists = [store.make_push_list(list(range(K)), d) for d in dev_sets]

    def do_step(i):
        store.push_list(lists[i % nsets])

    alg = cfg.algorithmic_bytes_per_step
    steps = int(max(30, min(20000, 0.4 / max(alg / 6.0e12, 4e-6))))      # about 0.4 s of launches
    for i in range(10):
        do_step(i)
    store.wait()
    store.timing_begin()
    t0 = time.perf_counter()
    for i in range(steps):
        do_step(i)
    store.wait()
    wall = time.perf_counter() - t0
    ev_ms, launches = store.timing_end()
    lps = launches / steps
    launch_s = ev_ms * 1e-3 / max(launches, 1)
    state_bytes = 16 * N
    out = {
        "workload": f"{cfg.name}: {K} keys, {N} params, W={cfg.W} {cfg.grad_dtype}, bucket {cfg.bucket_bytes} B",
        "data": f"gradients N(0, sigma_key) drawn on the GPU, {nsets} set(s) cycled",
        "steps": steps,
        "ms_per_step": round(wall / steps * 1e3, 5),
        "avg_launch_us": round(launch_s * 1e6, 3),
        "launches_per_step": lps,
        "units": store.plan.num_units,
        "value_GBps": round(N * cfg.W * cfg.grad_itemsize / (wall / steps) / 1e9, 2),
        "algorithmic_bytes_per_step": alg,
        "algorithmic_frac": round(alg / max(lps, 1e-9) / launch_s / 1e9 / HBM_PEAK_GBPS, 4),
        "tuning": store.get_tuning()[0],
    }
    if alg < (64 << 20):
        # the same steps issued by one native loop (kv_push_list_repeat): what a native caller sees, without the
        # interpreter and the ctypes call between two launches
        store.push_list_repeat(lists[0], 200)
        store.wait()
        store.timing_begin()
        t0 = time.perf_counter()
        store.push_list_repeat(lists[0], steps)
        store.wait()
        wall_native = time.perf_counter() - t0
        ev_native, launches_native = store.timing_end()
        out["native_loop_ms_per_step"] = round(wall_native / steps * 1e3, 5)
        out["native_loop_avg_launch_us"] = round(ev_native * 1e3 / max(launches_native, 1), 3)
        out["note"] = (f"launch bound and cache resident ({alg / 1e6:.1f} MB per step): the fraction says little; an empty "
                       f"kernel launch takes {floor_us:.2f} us on this box.  ms_per_step is a Python loop over the binding "
                       f"(one ctypes call per step); native_loop_* is the same list push repeated by one native call")
        out["launch_floor_us"] = round(floor_us, 3)
    if state_bytes // 2 > MALL_BYTES:
        out["cold_frac"] = out["algorithmic_frac"]
        out["cold_note"] = "w and m (%.0f MB) cannot stay in the 256 MiB memory-side cache: every step is a cold step" % (state_bytes / 2e6)
    else:
        cold = cold_leg(kv, store, do_step, cold_steps, evict_buf, False, alg)
        cold_d = cold_leg(kv, store, do_step, cold_steps, evict_buf, True, alg)
        if cold:
            out["cold_frac"] = cold["frac"]
            out["cold_avg_launch_us"] = cold["avg_launch_us"]
            out["cold_dirty_frac"] = cold_d["frac"]
            out["cold_dirty_avg_launch_us"] = cold_d["avg_launch_us"]
    store.close()
    del dev_sets, lists
    torch.cuda.empty_cache()
    return out


def cpu_baseline(cfg, weights, grads_host, seconds: float):
    """The oracle as it stands: (i) one thread, (ii) the same function on disjoint
    element ranges from one thread per host core."""
    from oracle import kv_oracle as orc
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    out = {}
    for label, threads in (("single", 1), ("all", cores)):
        st = orc.OracleStore(cfg.numel, cfg.W, lr=cfg.lr, momentum=cfg.momentum, wd=cfg.wd)
        for k, w in enumerate(weights):
            st.set_weights(k, w)
        st.step(grads_host, threads=threads)             # untimed first touch
        steps = 0
        t0 = time.perf_counter()
        while steps < 3 or time.perf_counter() - t0 < seconds:
            st.step(grads_host, threads=threads)
            steps += 1
        dt = (time.perf_counter() - t0) / steps
        out[label] = (threads, dt, steps)
    return out


def overlap_mode(args) -> int:
    """Overlap of aggregation with (synthetic) backward compute, the paper's actual claim.  The fused kernel can be
    confined to part of the chip (--workgroups-per-cu: a persistent grid of that many workgroups per compute unit)
    and the producers can leave wave slots free (--producer-workgroups) and be compute bound (--producer-bytes)."""
    import numpy as np
    import torch
    import workloads as wl
    import paper_1802_06949_amd as kv
    from paper_1802_06949_amd.engine import Engine
    from paper_1802_06949_amd.training_loop import EngineLoop

    cfg = wl.get_config(args.config)
    K, W = len(cfg.keys), cfg.W
    tdt = torch.float32 if cfg.grad_dtype == "f32" else torch.float16
    store = kv.KVStore(cfg.numel, W, cfg.grad_dtype, cfg.bucket_bytes, lr=cfg.lr, momentum=cfg.momentum, wd=cfg.wd,
                       descending=True, workgroups_per_cu=args.workgroups_per_cu, lane_elems=args.lane_elems,
                       unroll=args.unroll, resident_workgroups=args.resident_workgroups)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    staged = [(torch.randn(W, n, device="cuda", generator=gen) * 1e-3).to(tdt) for n in cfg.numel]
    live = [s.clone() for s in staged]                   # valid gradients even where a producer copies only a part
    side = torch.cuda.Stream()
    eng = Engine(args.engine_threads)
    biggest = max(cfg.numel)
    spin = [int(args.spin * n / biggest) for n in cfg.numel]
    loop = EngineLoop(store, eng, staged, live, side.cuda_stream, spin, max_workgroups=args.producer_workgroups,
                      copy_bytes_cap=args.producer_bytes)
    lists = store.make_push_list(list(range(K - 1, -1, -1)), [[live[k][r] for r in range(W)] for k in range(K - 1, -1, -1)])

    def timed(fn, reps):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e3

    def serial():
        loop.backward_only()
        side.synchronize()
        store.push_list(lists)
        store.wait()

    def overlapped():
        loop.step()
        store.wait()

    def one_launch_behind():
        # the producers of this iteration run while the ONE merged launch of the previous iteration's gradients does
        # (double-buffered gradients in a real loop; here the same buffers, which the producers rewrite with the same values)
        store.push_list(lists)
        loop.backward_only()
        side.synchronize()
        store.wait()

    reps = args.steps
    res = {
        "mode": "overlap",
        "workload": cfg.name,
        "spin": args.spin,
        "engine_threads": args.engine_threads,
        "producer_workgroups": args.producer_workgroups or 2048,
        "producer_bytes": args.producer_bytes or "all",
        "fused_workgroups_per_cu": store.get_tuning()[0]["workgroups_per_cu"],
        "backward_only_ms": round(timed(lambda: (loop.backward_only(), side.synchronize()), reps), 4),
        "aggregation_only_ms": round(timed(lambda: (store.push_list(lists), store.wait()), reps), 4),
        "serial_ms": round(timed(serial, reps), 4),
        "overlapped_ms": round(timed(overlapped, reps), 4),
        "merged_launch_beside_next_backward_ms": round(timed(one_launch_behind, reps), 4),
    }
    loop.close()
    eng.close()
    store.close()
    print(json.dumps(res))
    return 0


def main() -> int:
    args = parse_args()
    if args.steps <= 0:
        args.steps = 30 if args.overlap else 6000
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU only (the W gradient replicas sit in one MI355X's HBM); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import workloads as wl
    import paper_1802_06949_amd as kv

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    kv.load_library()                                   # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)
    if args.overlap:
        return overlap_mode(args)

    side = None
    if args.graph:
        if args.schedule != "chained" or args.sets > 7:
            print("--graph needs the chained schedule and at most 7 gradient sets", file=sys.stderr)
            return 2
        side = torch.cuda.Stream()          # the default stream cannot be captured
        torch.cuda.set_stream(side)
    cfg = wl.get_config(args.config)
    if args.ranks or args.grad_dtype:
        import dataclasses
        cfg = dataclasses.replace(cfg, W=args.ranks or cfg.W, grad_dtype=args.grad_dtype or cfg.grad_dtype,
                                  name=f"{cfg.name}[W={args.ranks or cfg.W},{args.grad_dtype or cfg.grad_dtype}]")
    K = len(cfg.keys)
    N = cfg.total_numel
    itemsize = cfg.grad_itemsize
    tdt = torch.float32 if cfg.grad_dtype == "f32" else torch.float16

    t_gen = time.perf_counter()
    weights = wl.make_weights(cfg, args.gen_threads)
    nsets = max(1, args.sets)
    host_sets = []
    dev_sets = []
    for s in range(nsets):
        g = wl.make_step_gradients(cfg, s, args.gen_threads)
        if args.flat_grads:
            offs, cur = [], 0
            for n in cfg.numel:
                offs.append(cur)
                cur += (n * itemsize + 255) // 256 * 256 // itemsize
            skew = args.rank_skew // itemsize
            voff = args.view_offset // itemsize
            flats = [torch.empty(cur + cfg.W * skew + voff, dtype=tdt, device="cuda")[r * skew + voff:] for r in range(cfg.W)]
            dset = []
            for k, gk in enumerate(g):
                row = []
                for r, a in enumerate(gk):
                    v = flats[r][offs[k]:offs[k] + a.size]
                    v.copy_(torch.from_numpy(a))
                    row.append(v)
                dset.append(row)
            dev_sets.append(dset)
        else:
            dev_sets.append([[torch.from_numpy(a).cuda() for a in gk] for gk in g])
        if s == 0:
            host_sets.append(g)
        del g
    t_gen = time.perf_counter() - t_gen

    store = kv.KVStore(cfg.numel, cfg.W, cfg.grad_dtype, cfg.bucket_bytes, lr=cfg.lr, momentum=cfg.momentum, wd=cfg.wd,
                       keep_sum=args.keep_sum, lazy=args.lazy, unroll=args.unroll, workgroups_per_cu=args.workgroups_per_cu,
                       nontemporal=args.nontemporal, xcd_remap=args.xcd_remap, lane_elems=args.lane_elems,
                       resident_workgroups=args.resident_workgroups, run_time_w=int(args.run_time_w), autotune=args.autotune)
    for k, w in enumerate(weights):
        if w.size:
            store.set_weights(k, torch.from_numpy(w).cuda())
    store.wait()
    bcast_bytes = 0
    if args.broadcast != "none":
        R = args.replicas or cfg.W
        rdt = torch.float32 if args.broadcast == "f32" else torch.float16
        reps = [[torch.empty(n, dtype=rdt, device="cuda") for _ in range(R)] for n in cfg.numel]
        for k in range(K):
            store.set_broadcast(k, reps[k], args.broadcast)
        bcast_bytes = N * R * (4 if args.broadcast == "f32" else 2)
    sched = {"chained": kv.KV_SCHED_CHAINED, "funnel": kv.KV_SCHED_FUNNEL, "concurrent": kv.KV_SCHED_CONCURRENT}[args.schedule]
    store.set_schedule(sched, args.streams, args.outstanding)
    keys = list(range(K))
    lists = [store.make_push_list(keys, d) for d in dev_sets]
    if args.push_mode == "each":
        # one kv_push per key, in key order, with the pointer arrays marshalled once
        import ctypes
        rows = [[(ctypes.c_void_p * cfg.W)(*[int(t.data_ptr()) for t in d[k]]) for k in keys] for d in dev_sets]
        raw_push, handle = store._L.kv_push, store._h

        def do_step(i):
            for k, row in enumerate(rows[i % nsets]):
                rc = raw_push(handle, k, row)
                if rc != 0:
                    raise kv.KVError(rc, store.last_error())
    else:
        def do_step(i):
            store.push_list(lists[i % nsets])

    for i in range(max(args.warmup, nsets if args.graph else 0, 45 if args.autotune else 0)):
        do_step(i)
    store.wait()
    torch.cuda.synchronize()
    launches_per_replay = 0
    if args.graph:
        eager_step, graphs = do_step, []
        for j in range(nsets):
            before = store.launch_log(0)[0]
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                eager_step(j)
            launches_per_replay = store.launch_log(0)[0] - before
            graphs.append(g)

        def do_step(i):
            graphs[i % nsets].replay()

    store.timing_begin()
    t0 = time.perf_counter()
    for i in range(args.steps):
        do_step(i)
    store.wait()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms, launches = store.timing_end()
    if args.graph:
        launches = args.steps * launches_per_replay       # the store counts a captured launch once, at capture

    # per-step times from a second, separate pass: an event after every step costs about 2 us per
    # step, so it stays out of the timed region above
    step_ms = []
    if args.schedule == "chained":
        store.timing_begin()
        for i in range(min(args.steps, 500)):
            do_step(i)
            store.timing_mark()
        store.wait()
        store.timing_end()
        step_ms = sorted(store.timing_intervals())

    t_step = wall / args.steps
    agg_gbps = N * cfg.W * itemsize / t_step / 1e9
    alg_bytes_step = cfg.algorithmic_bytes_per_step + bcast_bytes + (4 * N if args.keep_sum else 0)
    launches_per_step = launches / args.steps
    alg_bytes_launch = alg_bytes_step / max(launches_per_step, 1e-9)
    launch_s = ev_ms * 1e-3 / max(launches, 1)
    achieved = alg_bytes_launch / launch_s / 1e9

    extra = {}
    if args.pull_copy:
        outs = [torch.empty(n, dtype=torch.float32, device="cuda") for n in cfg.numel]
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for k in keys:
            store.pull(k, outs[k])
        store.wait()
        extra["pull_copy_all_keys_ms"] = (time.perf_counter() - t1) * 1e3
        store.pull_list(keys, outs)
        store.wait()
        t1 = time.perf_counter()
        for _ in range(20):
            store.pull_list(keys, outs)
        store.wait()
        extra["pull_list_all_keys_ms"] = (time.perf_counter() - t1) * 1e3 / 20

    props = torch.cuda.get_device_properties(0)
    device = {"name": props.name, "compute_units": props.multi_processor_count,
              "memory_GiB": round(props.total_memory / 2 ** 30, 1)}
    clk, width = getattr(props, "memory_clock_rate", None), getattr(props, "memory_bus_width", None)
    if clk and width:
        device["memory_clock_kHz"] = clk
        device["memory_bus_bits"] = width
        device["clock_x_width_x2_GBps"] = round(clk * 1e3 * width / 8 * 2 / 1e9, 1)     # double data rate
    extra["device"] = device
    if args.ceilings:
        # plain read and copy kernels on 1 GiB buffers (and on 96 MiB ones, which fit the memory-side
        # cache) as measured ceilings for context
        def rate(fn, nbytes_moved, reps=20):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return round(nbytes_moved * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)

        def filled(nb):
            t = torch.zeros(nb, dtype=torch.uint8, device="cuda")
            return t if args.ceilings_data == "zeros" else t.random_()

        ceil = {"data": args.ceilings_data}
        for label, nb in (("1GiB", 1 << 30), ("96MiB", 96 << 20)):
            a = filled(nb)
            b = filled(nb)
            ceil[f"read_{label}_GBps"] = rate(lambda: kv.read_bytes(a, nb), nb)
            ceil[f"copy_{label}_GBps"] = rate(lambda: kv.copy_bytes(b, a, nb), 2 * nb)
            del a, b
        # mixes of read and written streams of 512 MiB each with the fused kernel's access pattern (nothing
        # fits the memory-side cache), buffers as allocated and staggered by 4 KB per buffer
        per = 512 << 20
        pool = [filled(per + 64 * 4096) for _ in range(18)]
        for label, stagger in (("aligned", 0), ("staggered_4KB", 4096)):
            bufs = [b[i * stagger:i * stagger + per] for i, b in enumerate(pool)]
            for n_read, n_write in ((1, 0), (16, 0), (1, 1), (2, 2), (8, 8), (16, 1), (16, 2)):
                rd, wr = bufs[:n_read], bufs[n_read:n_read + n_write]
                ceil[f"mix_{n_read}r_{n_write}w_{label}_GBps"] = rate(lambda: kv.stream_mix(rd, wr, per),
                                                                     (n_read + n_write) * per, reps=10)
        del pool
        extra["ceilings"] = ceil

    if args.calib_copy > 0:
        nb = 1 << 30
        a = torch.empty(nb, dtype=torch.uint8, device="cuda")
        b = torch.empty(nb, dtype=torch.uint8, device="cuda")
        for _ in range(args.calib_copy):
            kv.copy_bytes(b, a, nb)
        torch.cuda.synchronize()
        extra["calib_copy_bytes"] = nb

    # cold-state legs of the headline workload, then the other configurations, all in this process
    traffic, traffic_source = read_traffic(cfg.name)
    cold = cold_dirty = None
    evict_buf = None
    plain = args.schedule == "chained" and not args.graph and args.broadcast == "none"
    if plain and (args.cold_steps > 0 or not args.no_other_configs):
        evict_buf = torch.zeros(EVICT_BYTES // 4, dtype=torch.float32, device="cuda")
    if plain and args.cold_steps > 0:
        if args.cold_evict in ("both", "clean"):
            cold = cold_leg(kv, store, do_step, args.cold_steps, evict_buf, False, alg_bytes_step)
        if args.cold_evict in ("both", "dirty"):
            cold_dirty = cold_leg(kv, store, do_step, args.cold_steps, evict_buf, True, alg_bytes_step)
    floor_us = launch_floor_us(kv)
    state_bytes = 8 * N
    grad_bytes = N * cfg.W * itemsize

    result = {
        "metric": METRIC,
        "value": round(agg_gbps, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(t_step * 1e3, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {
            "workload": f"{cfg.name}: {K} keys, {N} params, W={cfg.W} {cfg.grad_dtype} gradient copies, "
                        f"bucket {cfg.bucket_bytes} B, lr={cfg.lr} momentum={cfg.momentum} wd={cfg.wd}",
            "gradient_sets_cycled": nsets,
            "units": store.plan.num_units,
            "launches_per_step": launches_per_step,
            "push_mode": args.push_mode + (", replayed from HIP graphs" if args.graph else ""),
            "tuning": dict(store.get_tuning()[0], self_tuned=args.autotune, settled=store.get_tuning()[1],
                           wide_launches=store.wide_launches()),
            "schedule": args.schedule + (f" ({args.streams} streams, barrier every {args.outstanding} keys)"
                                         if args.schedule == "concurrent" else ""),
            "pull": "zero-copy (weights read in place in the arena)" if args.broadcast == "none" else
                    f"fused broadcast to {args.replicas or cfg.W} {args.broadcast} replicas per key (+{bcast_bytes} B per step)",
        },
        "params_per_s": round(N / t_step, 1),
        "algorithmic_hbm_GBps": round(alg_bytes_step / t_step / 1e9, 2),
        "algorithmic_hbm_frac_of_peak": round(alg_bytes_step / t_step / 1e9 / HBM_PEAK_GBPS, 4),
        "roofline": {
            "bound": "hbm",
            "kernel": "kv_fused",
            "achieved": round(achieved, 2),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": traffic,
            "traffic_source": traffic_source,
            "algorithmic_bytes_per_launch": alg_bytes_launch,
            "avg_launch_us": round(launch_s * 1e6, 3),
            "median_step_us_with_event_per_step": round(step_ms[len(step_ms) // 2] * 1e3, 3) if step_ms else None,
            "min_step_us_with_event_per_step": round(step_ms[0] * 1e3, 3) if step_ms else None,
            "launches_timed": launches,
            "state_residency": (
                f"steps run back to back: the {state_bytes / 1e6:.0f} MB of w and m fit the 256 MiB memory-side cache and stay "
                f"there between launches, so {2 * state_bytes / alg_bytes_step:.0%} of the algorithmic bytes (w, m read and "
                f"written) never reach DRAM; DRAM itself delivers the {grad_bytes / 1e6:.0f} MB of gradients per launch "
                f"({grad_bytes / launch_s / 1e9:.0f} GB/s, {grad_bytes / launch_s / 1e9 / HBM_PEAK_GBPS:.0%} of peak); "
                "roofline.cold has the same launch with the state evicted" if state_bytes <= MALL_BYTES else
                f"the {state_bytes / 1e6:.0f} MB of w and m do not fit the 256 MiB memory-side cache: every launch reads "
                "and writes them in DRAM"),
            "cold": cold,
            "cold_dirty": cold_dirty,
        },
        "launch_floor_us": round(floor_us, 3),
    }
    result.update(extra)
    if plain and not args.no_other_configs:
        others = []
        for cid in (1, 2, 4, 5, 6):
            if cid != args.config:
                others.append(other_config_leg(kv, cid, evict_buf, args.cold_steps, floor_us))
        result["other_configs"] = others
    del evict_buf

    if not args.no_cpu_baseline:
        base = cpu_baseline(cfg, weights, host_sets[0], args.cpu_seconds)
        threads, dt, cpu_steps = base["all"]
        result["cpu_baseline"] = {
            "value": round(N * cfg.W * itemsize / dt / 1e9, 3),
            "unit": "GB/s",
            "cores": threads,
            "kind": "oracle",
            "sample": f"{cpu_steps} full steps of the same workload (all {K} keys, one gradient set), after one "
                      f"untimed step; the single-thread leg ran {base['single'][2]} steps.  The all-core leg is the "
                      "unmodified oracle: it cuts each key into one element range per core with a thread pool made per "
                      "key, and runs keys below 4096 elements per core on one thread, so it does not scale with the cores",
            "ms_per_step": round(dt * 1e3, 2),
            "single_thread_value": round(N * cfg.W * itemsize / base["single"][1] / 1e9, 3),
            "single_thread_ms_per_step": round(base["single"][1] * 1e3, 2),
        }
    result["input_generation_s"] = round(t_gen, 2)
    store.close()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
