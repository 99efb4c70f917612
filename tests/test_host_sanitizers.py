"""Host-side sanitizer runs (CPU only): the bucket plan, tiling and launch chain under
AddressSanitizer + UBSan, the dependency engine under ThreadSanitizer, the C oracle under
AddressSanitizer + UBSan, each driven by a small random-input program in tests/native/."""
from __future__ import annotations

import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")
CSRC = os.path.join(ROOT, "paper_1802_06949_amd", "csrc")
INC = os.path.join(ROOT, "include")
HIP_INC = "/opt/rocm/include"

pytestmark = pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")


def _build_and_run(tmp_path, name, cmd, env=None):
    exe = str(tmp_path / name)
    r = subprocess.run(cmd + ["-o", exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    return r.stdout


def test_plan_tiles_and_chain_under_asan_ubsan(tmp_path):
    out = _build_and_run(tmp_path, "plan_chain_fuzz",
                         ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                          "-I", CSRC, "-I", INC, os.path.join(NATIVE, "plan_chain_fuzz.cpp"), os.path.join(CSRC, "kv_plan.cpp")])
    assert "ok" in out


def test_oracle_under_asan_ubsan(tmp_path):
    out = _build_and_run(tmp_path, "oracle_fuzz",
                         ["gcc", "-std=c99", "-O1", "-g", "-ffp-contract=off", "-fsanitize=address,undefined",
                          "-fno-sanitize-recover=undefined", os.path.join(NATIVE, "oracle_fuzz.c"),
                          os.path.join(ROOT, "oracle", "kv_oracle.c")])
    assert "ok" in out


@pytest.mark.skipif(not os.path.exists(os.path.join(HIP_INC, "hip", "hip_runtime_api.h")), reason="needs the HIP headers")
def test_store_steady_state_allocates_nothing(tmp_path):
    """The whole host side of the store (kv_store.cpp + kv_plan.cpp) against a stand-in HIP runtime, under
    AddressSanitizer + UBSan, with every operator new and every allocating runtime call counted."""
    out = _build_and_run(tmp_path, "alloc_count",
                         ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                          "-D__HIP_PLATFORM_AMD__", "-I", HIP_INC, "-I", CSRC, "-I", INC,
                          os.path.join(NATIVE, "alloc_count.cpp"), os.path.join(NATIVE, "hip_stub.cpp"),
                          os.path.join(CSRC, "kv_store.cpp"), os.path.join(CSRC, "kv_plan.cpp")])
    assert "allocates nothing: ok" in out


@pytest.mark.skipif(not os.path.exists(os.path.join(HIP_INC, "hip", "hip_runtime_api.h")), reason="needs the HIP headers")
def test_engine_under_thread_sanitizer(tmp_path):
    env = dict(os.environ, LD_LIBRARY_PATH="/opt/rocm/lib:" + os.environ.get("LD_LIBRARY_PATH", ""))
    out = _build_and_run(tmp_path, "engine_fuzz",
                         ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=thread", "-D__HIP_PLATFORM_AMD__", "-I", HIP_INC,
                          "-I", CSRC, "-I", INC, os.path.join(NATIVE, "engine_fuzz.cpp"), os.path.join(CSRC, "kv_engine.cpp"),
                          "-L/opt/rocm/lib", "-lamdhip64", "-pthread"], env=env)
    assert "ok" in out
