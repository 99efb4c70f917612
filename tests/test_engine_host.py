"""CPU tests of the dependency engine against a sequential oracle: operations run
in push order by a plain loop must leave the same values as the engine's
concurrent execution, for any pattern of read and mutate sets (the paper's
Dependency Tracking section); plus the ordering properties it states."""
from __future__ import annotations

import threading
import time

import numpy as np
import pytest

kv = pytest.importorskip("paper_1802_06949_amd")
from paper_1802_06949_amd.engine import Engine  # noqa: E402


def _rng(*seed):
    return np.random.Generator(np.random.SFC64(list(seed)))


def test_paper_example_b_equals_a_plus_one():
    """Engine.push(lambda: b.data = a.data + 1, read=[a.tag], mutate=[b.tag])"""
    eng = Engine(2)
    a, b = eng.new_var(), eng.new_var()
    data = {"a": 0, "b": 0}
    eng.push(lambda: data.__setitem__("a", 41), mutate=[a])
    eng.push(lambda: data.__setitem__("b", data["a"] + 1), read=[a], mutate=[b])
    eng.wait_var(b)
    assert data["b"] == 42
    eng.close()


@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("threads", [1, 4, 16])
def test_random_programs_match_sequential_execution(seed, threads):
    r = _rng(5, seed)
    V, N = int(r.integers(1, 9)), 300
    prog = []
    for i in range(N):
        reads = [int(x) for x in r.choice(V, size=int(r.integers(0, min(V, 3) + 1)), replace=False)]
        writes = [int(x) for x in r.choice(V, size=int(r.integers(0, min(V, 2) + 1)), replace=False)]
        prog.append((i, reads, writes))

    def run_op(vals, i, reads, writes):
        acc = i + 1
        for v in reads:
            acc = (acc * 1000003 + vals[v]) % 2147483647
        for v in writes:
            vals[v] = (vals[v] * 31 + acc) % 2147483647

    ref = [0] * V                                   # the oracle: a plain loop in push order
    for i, reads, writes in prog:
        run_op(ref, i, reads, writes)

    vals = [0] * V
    eng = Engine(threads)
    tags = [eng.new_var() for _ in range(V)]
    for i, reads, writes in prog:
        eng.push(lambda i=i, reads=reads, writes=writes: run_op(vals, i, reads, writes),
                 read=[tags[v] for v in reads], mutate=[tags[v] for v in writes])
    eng.wait_all()
    assert vals == ref
    assert eng.stats()[0] == N
    eng.close()


def test_writes_to_one_variable_run_in_push_order_one_at_a_time():
    """The property the paper uses to order its collectives (the dummy variable)."""
    eng = Engine(8)
    dummy = eng.new_var()
    log, active, worst = [], [0], [0]
    lock = threading.Lock()

    def op(i):
        with lock:
            active[0] += 1
            worst[0] = max(worst[0], active[0])
        time.sleep(0.0005)
        log.append(i)
        with lock:
            active[0] -= 1

    for i in range(100):
        eng.push(lambda i=i: op(i), mutate=[dummy])
    eng.wait_var(dummy)
    assert log == list(range(100)) and worst[0] == 1
    eng.close()


def test_consecutive_reads_run_together_and_fence_the_next_write():
    eng = Engine(4)
    x = eng.new_var()
    both_in = threading.Barrier(3, timeout=10)      # only passable if three readers are inside at once
    state = {"readers_done": 0, "writer_saw": None}
    lock = threading.Lock()

    def reader():
        both_in.wait()
        time.sleep(0.01)
        with lock:
            state["readers_done"] += 1

    def writer():
        state["writer_saw"] = state["readers_done"]

    eng.push(lambda: None, mutate=[x])
    for _ in range(3):
        eng.push(reader, read=[x])
    eng.push(writer, mutate=[x])
    eng.wait_all()
    assert state["writer_saw"] == 3                 # the write waited for every read before it
    assert eng.stats()[1] >= 3
    eng.close()


def test_independent_variables_do_not_wait_for_each_other():
    eng = Engine(2)
    a, b = eng.new_var(), eng.new_var()
    gate = threading.Event()
    out = []
    eng.push(lambda: gate.wait(10), mutate=[a])      # blocks variable a
    eng.push(lambda: out.append("b"), mutate=[b])    # must not be held up by it
    eng.wait_var(b)
    assert out == ["b"]
    gate.set()
    eng.wait_all()
    eng.close()


def test_bad_arguments():
    eng = Engine(1)
    v = eng.new_var()
    with pytest.raises(kv.KVError) as e:
        eng.push(lambda: None, read=[v + 5])
    assert e.value.status == -2
    with pytest.raises(kv.KVError):
        eng.wait_var(99)
    with pytest.raises(kv.KVError):
        Engine(0)
    eng.close()
