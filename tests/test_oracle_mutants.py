"""Do the pins notice a mistake?  Each case plants ONE plausible mistake (a dropped term, a wrong sign, a wrong
operand, another summation order, a fused rounding, a wrong rounding rule) in a copy of the oracle's C source,
builds it, and runs the oracle's pins against that build.  At least one pin has to fail.

The pins are run WITHOUT the numpy float32 cross-check, which re-types the oracle's formulas and therefore does not
count as a pin: hand-computed cases, closed forms, exactness properties and library routines have to do the job.
CPU only; nothing here touches the GPU library.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

from oracle import build as obuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# (name, text in kv_oracle.c that occurs exactly once, replacement)
MUTANTS = [
    ("left_fold_starts_from_zero",
     "float s = v[0];\n    for (int r = 1; r < W; ++r) s = s + v[r];",
     "float s = 0.0f;\n    for (int r = 0; r < W; ++r) s = s + v[r];"),
    ("left_fold_runs_from_the_last_rank",
     "float s = v[0];\n    for (int r = 1; r < W; ++r) s = s + v[r];",
     "float s = v[W - 1];\n    for (int r = W - 2; r >= 0; --r) s = s + v[r];"),
    ("left_fold_is_a_tree",
     "return order == KVO_PAIRWISE ? fold_pairwise(v, 0, W) : fold_sequential(v, W);",
     "return fold_pairwise(v, 0, W);"),
    ("tree_is_a_left_fold",
     "return order == KVO_PAIRWISE ? fold_pairwise(v, 0, W) : fold_sequential(v, W);",
     "return fold_sequential(v, W);"),
    ("tree_splits_in_the_middle",
     "while (2 * h < n) h *= 2;",
     "h = n / 2;"),
    ("tree_split_not_strictly_below",
     "while (2 * h < n) h *= 2;",
     "while (4 * h < n) h *= 2;"),
    ("every_rank_reads_rank_zero",
     "else                  v[r] = ((const float*)grads[r])[i];",
     "else                  v[r] = ((const float*)grads[0])[i];"),
    ("scale_dropped",
     "float ghat = rescale * s;",
     "float ghat = s;"),
    ("scale_by_division_of_the_inverse",
     "float ghat = rescale * s;",
     "float ghat = s / (1.0f / rescale);"),
    ("weight_decay_dropped",
     "float wdw = wd * w[i];",
     "float wdw = 0.0f * w[i];"),
    ("weight_decay_sign",
     "float t = ghat + wdw;",
     "float t = ghat - wdw;"),
    ("weight_decay_on_momentum",
     "float wdw = wd * w[i];",
     "float wdw = wd * m[i];"),
    ("weight_decay_outside_the_learning_rate",
     "float lt = lr * t;",
     "float lt = lr * ghat + wdw;"),
    ("momentum_dropped",
     "float mm = momentum * m[i];",
     "float mm = 0.0f * m[i];"),
    ("gradient_sign",
     "float dw = mm - lt;",
     "float dw = mm + lt;"),
    ("state_keeps_the_scaled_gradient",
     "m[i] = dw;",
     "m[i] = -lt;"),
    ("weights_move_by_old_momentum",
     "float wn = w[i] + dw;",
     "float wn = w[i] + mm - lr * ghat;"),
    ("learning_rate_on_momentum_too",
     "float dw = mm - lt;",
     "float dw = lr * (mm - t);"),
    ("raw_sum_is_stored_scaled",
     "if (sum_out) sum_out[i] = s;",
     "if (sum_out) sum_out[i] = ghat;"),
    ("half_normal_rebias",
     "bits = sign | ((e + 112u) << 23) | (f << 13);",
     "bits = sign | ((e + 111u) << 23) | (f << 13);"),
    ("half_subnormal_exponent",
     "bits = sign | ((uint32_t)(113 - shift) << 23) | (f << 13);",
     "bits = sign | ((uint32_t)(112 - shift) << 23) | (f << 13);"),
    ("half_subnormal_flushed",
     "} else if (f == 0) {                    /* signed zero */",
     "} else if (f == 0 || e == 0) {          /* signed zero */"),
    ("to_half_ties_round_up",
     "if (rem > 0x1000u || (rem == 0x1000u && (q & 1u))) ++q;   /* a carry runs into the exponent */",
     "if (rem >= 0x1000u) ++q;"),
    ("to_half_truncates",
     "if (rem > 0x1000u || (rem == 0x1000u && (q & 1u))) ++q;   /* a carry runs into the exponent */",
     ""),
    ("to_half_largest_half_overflows",
     "if (a >= 0x477FF000u) return",
     "if (a >= 0x477FE000u) return"),
    ("to_half_subnormal_ties_round_up",
     "if (rem > half || (rem == half && (q & 1u))) ++q;",
     "if (rem >= half) ++q;"),
    ("to_half_small_values_flushed",
     "if (a < 0x33000000u) return sign;",
     "if (a < 0x38800000u) return sign;"),
]

# the same source, built with fused multiply-adds allowed: two roundings become one
FUSED = "fused_multiply_add"

PIN_CMD = [sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q", "-p", "no:cacheprovider",
           "-k", "not numpy_float32_cross_check"]


def _host_has_fma() -> bool:
    try:
        with open("/proc/cpuinfo") as f:
            return " fma " in f.read().replace("\n", " ")
    except OSError:
        return False


def _build(src_text: str, out: str, cflags) -> None:
    c = out[:-3] + ".c"
    with open(c, "w") as f:
        f.write(src_text)
    subprocess.run(["gcc", *cflags, "-o", out, c], check=True)


def _run_pins(lib: str):
    env = dict(os.environ, KVO_LIBRARY=lib)
    r = subprocess.run(PIN_CMD, cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
    return r.returncode, r.stdout[-1500:]


@pytest.fixture(scope="module")
def verdicts(tmp_path_factory):
    """Builds every mutant and runs the pins against each, four at a time."""
    d = tmp_path_factory.mktemp("mutants")
    with open(obuild.SRC) as f:
        src = f.read()
    libs = {}
    for name, old, new in MUTANTS:
        assert src.count(old) == 1, f"mutant {name}: its anchor text must occur exactly once in kv_oracle.c"
        libs[name] = str(d / f"{name}.so")
        _build(src.replace(old, new), libs[name], obuild.CFLAGS)
    libs["unchanged"] = str(d / "unchanged.so")
    _build(src, libs["unchanged"], obuild.CFLAGS)
    if _host_has_fma():
        libs[FUSED] = str(d / f"{FUSED}.so")
        flags = [f for f in obuild.CFLAGS if f != "-ffp-contract=off"] + ["-ffp-contract=fast", "-mfma"]
        _build(src, libs[FUSED], flags)
    with ThreadPoolExecutor(4) as ex:
        return dict(zip(libs, ex.map(_run_pins, libs.values())))


def test_the_unchanged_copy_passes_every_pin(verdicts):
    rc, tail = verdicts["unchanged"]
    assert rc == 0, tail


@pytest.mark.parametrize("name", [m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(verdicts, name):
    rc, tail = verdicts[name]
    assert rc == 1 and " failed" in tail, f"no pin noticed the mistake '{name}' (pytest exit code {rc})\n{tail}"


def test_fused_rounding_fails_a_pin(verdicts):
    if FUSED not in verdicts:
        pytest.skip("host has no fused multiply-add instruction")
    rc, tail = verdicts[FUSED]
    assert rc == 1 and " failed" in tail, f"no pin noticed fused multiply-adds\n{tail}"


# ------------------------------------------------------------------ the bucket-packing scan (Python)
PACKER_MUTANTS = [
    ("key_of_exactly_one_bucket_is_small", "if size >= bucket_bytes:", "if size > bucket_bytes:"),
    ("exact_fit_is_refused", "open_bytes + size <= bucket_bytes", "open_bytes + size < bucket_bytes"),
    ("large_key_closes_the_open_bucket",
     "units.append(Unit([k], True))\n            continue",
     "units.append(Unit([k], True))\n            open_unit = None\n            continue"),
    ("size_ignores_the_gradient_dtype", "size = int(n) * grad_itemsize", "size = int(n) * 4"),
    ("new_bucket_keeps_the_old_byte_count", "open_bytes = size\n", "open_bytes += size\n"),
    ("bucket_never_closes", "open_unit is not None and open_bytes + size <= bucket_bytes", "open_unit is not None"),
    ("keys_not_aligned_in_the_arena", "cur = (cur + align_elems - 1) // align_elems * align_elems", "pass"),
    ("arena_in_key_order",
     "for u in units:\n        for k in u.keys:\n            cur =",
     "for u in [Unit(list(range(len(numel))), False)]:\n        for k in u.keys:\n            cur ="),
]


def _packer_pins():
    """Calls every test of the packer's pin module in this process (its parametrised ones once per case)."""
    import tests.test_oracle_packer as pins
    for name, fn in sorted(vars(pins).items()):
        if not name.startswith("test_") or not callable(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            fn()
            continue
        names = [n.strip() for n in marks[0].args[0].split(",")]
        for values in marks[0].args[1]:
            fn(**dict(zip(names, values)))


def test_the_unchanged_packer_passes_its_pins():
    _packer_pins()


@pytest.mark.parametrize("name,old,new", PACKER_MUTANTS, ids=[m[0] for m in PACKER_MUTANTS])
def test_a_planted_packer_mistake_fails_a_pin(monkeypatch, name, old, new):
    import inspect

    from oracle import kv_oracle as orc
    src = inspect.getsource(orc.plan_units) + "\n\n" + inspect.getsource(orc.arena_offsets)
    assert src.count(old) == 1, f"mutant {name}: its anchor text must occur exactly once"
    scope = dict(vars(orc))
    exec(compile(src.replace(old, new), f"<mutant {name}>", "exec"), scope)
    monkeypatch.setattr(orc, "plan_units", scope["plan_units"])
    monkeypatch.setattr(orc, "arena_offsets", scope["arena_offsets"])
    with pytest.raises(AssertionError):
        _packer_pins()
