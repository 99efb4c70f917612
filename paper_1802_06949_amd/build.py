"""Builds libkv_mi355x.so (HIP kernels + C ABI) for gfx950 with hipcc.

The fused kernel source is compiled once per (gradient dtype, W) pair so that
the instantiations build in parallel; all objects are linked into one shared
library that sits next to this file.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libkv_mi355x.so")

FUSED_W = (0, 2, 4, 8, 16, 32)

COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra", "-Wno-unused-parameter"]
# Bit parity with the definition needs one rounding per operation and subnormals
# kept.  Packed fp32 instructions are switched off as a precaution against
# miscompiled forms on this hardware generation.
DEVICE = ["--offload-arch=gfx950", "-ffp-contract=off", "-fno-fast-math", "-fno-gpu-flush-denormals-to-zero",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def _jobs():
    jobs = []
    for f16 in (0, 1):
        for w in FUSED_W:
            jobs.append((os.path.join(CSRC, "kv_fused.hip"), os.path.join(OBJ, f"kv_fused_f{f16}_w{w}.o"),
                         DEVICE + [f"-DKV_TU_F16={f16}", f"-DKV_TU_W={w}"]))
    jobs.append((os.path.join(CSRC, "kv_dispatch.hip"), os.path.join(OBJ, "kv_dispatch.o"), DEVICE))
    jobs.append((os.path.join(CSRC, "kv_static.hip"), os.path.join(OBJ, "kv_static.o"), DEVICE))
    jobs.append((os.path.join(CSRC, "kv_plan.cpp"), os.path.join(OBJ, "kv_plan.o"), []))
    jobs.append((os.path.join(CSRC, "kv_store.cpp"), os.path.join(OBJ, "kv_store.o"), []))
    jobs.append((os.path.join(CSRC, "kv_diag.cpp"), os.path.join(OBJ, "kv_diag.o"), []))
    jobs.append((os.path.join(CSRC, "kv_engine.cpp"), os.path.join(OBJ, "kv_engine.o"), []))
    return jobs


def _deps():
    inc = os.path.join(HERE, "..", "include")
    return [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(inc, f) for f in os.listdir(inc)]


def build(force: bool = True, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hipcc = _hipcc()
    newest = max(os.path.getmtime(p) for p in _deps())
    todo = []
    for src, obj, extra in _jobs():
        if force or not os.path.exists(obj) or os.path.getmtime(obj) < newest:
            todo.append([hipcc, *COMMON, *extra, "-c", src, "-o", obj])

    def run(cmd):
        r = subprocess.run(cmd, capture_output=True, text=True)
        if verbose or r.returncode != 0:
            sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + r.stderr)
        if r.returncode != 0:
            raise RuntimeError("compile failed: " + cmd[-3])
        return r

    workers = max(1, min(8, os.cpu_count() or 1))
    with ThreadPoolExecutor(workers) as ex:
        list(ex.map(run, todo))
    objs = [obj for _, obj, _ in _jobs()]
    if todo or not os.path.exists(LIB):
        tmp = LIB + f".tmp{os.getpid()}"
        run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-o", tmp, *objs])
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose="-v" in sys.argv))
