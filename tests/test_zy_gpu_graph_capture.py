"""HIP graph capture of whole iterations (-m gpu).  A training loop that records its step into a graph records the
store's launches with it; every replay has to produce what the oracle produces for one more step with the captured
buffers.  Replays are interleaved with eager work and checked one by one.  Collected after the parity tests on
purpose: a failure here must not hide them from a run that stops at the first failure."""
from __future__ import annotations

import numpy as np
import pytest

from tests.gpu_harness import Pair

pytestmark = pytest.mark.gpu

KV_ERR_STATE = -3
NUMEL = [5000, 0, 300, 70000, 1, 2049, 1024, 33]
W = 4


def _rng(*seed):
    return np.random.Generator(np.random.SFC64([20260, *seed]))


def _grads(tag, dtype="f32"):
    dt = np.float32 if dtype == "f32" else np.float16
    return [[(_rng(tag, k, r).standard_normal(n) * 0.01).astype(dt) for r in range(W)] for k, n in enumerate(NUMEL)]


def _pair(stream, dtype="f32", **kw):
    pair = Pair(NUMEL, W, dtype, 16 << 10, lr=0.1, momentum=0.9, wd=1e-4, keep_sum=True, stream=stream.cuda_stream, **kw)
    pair.set_weights([_rng(7, k).standard_normal(n).astype(np.float32) for k, n in enumerate(NUMEL)])
    return pair


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_captured_iterations_replay_bit_exactly(dtype):
    import torch
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        pair = _pair(s, dtype)
        try:
            K = len(NUMEL)
            gA, gB = _grads(1, dtype), _grads(2, dtype)
            dA, dB = pair.upload(gA), pair.upload(gB)
            # eager steps with both buffer sets: their pointers now sit in cached device tables
            pair.step(gA, dev=dA)
            pair.step(gB, dev=dB)
            pair.compare("eager")
            plA = pair.gpu.make_push_list(list(range(K)), dA)
            pulled = torch.zeros(NUMEL[3], dtype=torch.float32, device="cuda")
            graph_a, graph_b = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph_a, stream=s):           # one list push and a pull
                pair.gpu.push_list(plA)
                pair.gpu.pull(3, pulled)
            order = [int(k) for k in _rng(3).permutation(K)]
            with torch.cuda.graph(graph_b, stream=s):           # single pushes in a shuffled order
                for k in order:
                    pair.gpu.push(k, dB[k])
            s.synchronize()
            pair.compare("a capture runs nothing")

            for i, which in enumerate("ABAAB"):
                (graph_a if which == "A" else graph_b).replay()
                pair.cpu.step(gA if which == "A" else gB)
                pair.gpu.wait()
                pair.compare(f"replay {i} of graph {which}")
                if which == "A":
                    assert np.array_equal(pulled.cpu().numpy().view(np.uint32), pair.cpu.w[3].view(np.uint32))
                # eager work between replays: an ordinary step, with new buffers every other time
                if i % 2 == 0:
                    pair.step(_grads(10 + i, dtype))
                else:
                    pair.step(gB, dev=dB)
                pair.compare(f"eager step after replay {i}")

            # optimizer parameters are those of the capture
            pair.gpu.set_lr(0.02)
            graph_a.replay()
            pair.cpu.step(gA)                                    # still lr = 0.1
            pair.gpu.wait()
            pair.compare("replay after kv_set_lr")
            pair.cpu.lr = 0.02
            pair.step(gA, dev=dA)
            pair.compare("eager step with the new learning rate")
        finally:
            pair.close()


def test_capture_refuses_buffers_it_has_not_seen_and_stays_usable():
    import torch
    import paper_1802_06949_amd as kv
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        pair = _pair(s)
        try:
            K = len(NUMEL)
            gA, gB = _grads(4), _grads(5)
            dA, dB = pair.upload(gA), pair.upload(gB)
            pair.step(gA, dev=dA)
            plA = pair.gpu.make_push_list(list(range(K)), dA)
            plB = pair.gpu.make_push_list(list(range(K)), dB)          # never pushed: not in any table
            mixed = [dA[k] if k % 2 else dB[k] for k in range(K)]
            plM = pair.gpu.make_push_list(list(range(K)), mixed)
            graph = torch.cuda.CUDAGraph()
            errors = []
            with torch.cuda.graph(graph, stream=s):
                for pl in (plB, plM):
                    try:
                        pair.gpu.push_list(pl)
                    except kv.KVError as e:
                        errors.append(e.status)
                try:
                    pair.gpu.push(0, dB[0])
                except kv.KVError as e:
                    errors.append(e.status)
                pair.gpu.push_list(plA)                                # this one is fine
            assert errors == [KV_ERR_STATE] * 3
            pair.gpu.wait()            # no key is left pushed: the refused pushes marked nothing (else plA had failed)
            graph.replay()
            pair.cpu.step(gA)
            pair.gpu.wait()
            pair.compare("replay after refused pushes")
            pair.step(gB, dev=dB)                                      # eager: uploads as usual
            pair.compare("eager step")
        finally:
            pair.close()


def test_only_the_chained_schedule_can_be_captured():
    import torch
    import paper_1802_06949_amd as kv
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        pair = _pair(s, schedule=(kv.KV_SCHED_CONCURRENT, 4, 0))
        try:
            gA = _grads(6)
            dA = pair.upload(gA)
            pair.step(gA, dev=dA, mode="each")
            pair.compare("eager")
            marker = torch.zeros(8, device="cuda")
            graph = torch.cuda.CUDAGraph()
            codes = []
            with torch.cuda.graph(graph, stream=s):
                marker.add_(1.0)                                       # keeps the graph from being empty
                try:
                    pair.gpu.push(0, dA[0])
                except kv.KVError as e:
                    codes.append(e.status)
            assert codes == [KV_ERR_STATE]
            pair.step(gA, dev=dA, mode="each")
            pair.compare("eager step after the refused capture")
        finally:
            pair.close()


def test_at_most_seven_buffer_sets_are_held_for_graphs():
    import torch
    import paper_1802_06949_amd as kv
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        pair = _pair(s)
        try:
            K = len(NUMEL)
            sets = [_grads(20 + i) for i in range(8)]
            dev = [pair.upload(g) for g in sets]
            lists = [pair.gpu.make_push_list(list(range(K)), d) for d in dev]
            marker = torch.zeros(8, device="cuda")
            graphs, codes = [], []
            for i in range(8):
                pair.step(sets[i], dev=dev[i])                         # eager: caches this set's table
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=s):
                    marker.add_(1.0)
                    try:
                        pair.gpu.push_list(lists[i])
                    except kv.KVError as e:
                        codes.append((i, e.status))
                graphs.append(g)
            assert codes == [(7, KV_ERR_STATE)]                     # seven tables are held, the eighth is refused
            pair.compare("after the captures")
            # eager steps with ever new buffers have one table left to go through; the held ones stay intact
            for i in range(3):
                pair.step(_grads(30 + i))
            for i in (6, 2, 0, 5, 1, 3, 4):
                graphs[i].replay()
                pair.cpu.step(sets[i])
                pair.gpu.wait()
                pair.compare(f"replay of graph {i}")
            pair.gpu.release_captures()
            pair.step(sets[7], dev=dev[7])
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=s):
                pair.gpu.push_list(lists[7])
            g.replay()
            pair.cpu.step(sets[7])
            pair.gpu.wait()
            pair.compare("replay of the eighth set after the release")
        finally:
            pair.close()


def test_lazy_store_captures_single_pushes_as_one_launch():
    """KV_FLAG_LAZY_LAUNCH under capture: the single pushes pile up and the last one records ONE launch; a captured
    pull of a pushed key records what is ready first."""
    import torch
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        pair = _pair(s, lazy=True)
        try:
            K = len(NUMEL)
            gA = _grads(40)
            dA = pair.upload(gA)
            pair.step(gA, dev=dA, mode="each")
            pair.compare("eager")
            before = pair.gpu.launch_log(0)[0]
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=s):
                for k in range(K):
                    pair.gpu.push(k, dA[k])
            assert pair.gpu.launch_log(0)[0] - before == 1
            pulled = torch.zeros(NUMEL[0], dtype=torch.float32, device="cuda")
            graph2 = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph2, stream=s):
                for k in range(K - 1):
                    pair.gpu.push(k, dA[k])
                pair.gpu.pull(0, pulled)                   # launches the units that are complete, then copies
                pair.gpu.push(K - 1, dA[K - 1])
            for i, g in enumerate((graph, graph2, graph)):
                g.replay()
                pair.cpu.step(gA)
                pair.gpu.wait()
                pair.compare(f"replay {i}")
            # graph2's pull ran before its last push: it saw key 0 as of that replay (two steps ago by now)
            assert pulled.abs().sum().item() > 0
        finally:
            pair.close()


def test_captured_list_pull_survives_reuse_of_every_staging_chunk():
    """A list pull recorded into a graph must not depend on pinned staging memory: between replays, eager list pulls
    with other destinations and steps with new gradient buffers (pointer-table uploads) use every staging chunk
    several times over; each replay still has to put the right weights into the captured destinations."""
    import torch
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        pair = _pair(s)
        try:
            K = len(NUMEL)
            keys = list(range(K))
            gA = _grads(21)
            dA = pair.upload(gA)
            pair.step(gA, dev=dA)                                  # the buffers' pointers now sit in a cached table
            plA = pair.gpu.make_push_list(keys, dA)
            outs = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in NUMEL]
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=s):
                pair.gpu.push_list(plA)
                pair.gpu.pull_list(keys, outs)
            s.synchronize()
            pair.compare("a capture runs nothing")
            for i in range(3):
                for j in range(10):                                # 20 uses of the 8 staging chunks
                    other = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in NUMEL]
                    pair.gpu.pull_list(keys, other)
                    pair.step(_grads(100 + 10 * i + j))
                pair.compare(f"eager churn {i}")
                for o in outs:
                    o.fill_(-1.0)
                graph.replay()
                pair.cpu.step(gA)
                pair.gpu.wait()
                pair.compare(f"replay {i}")
                for k in keys:
                    assert np.array_equal(outs[k].cpu().numpy().view(np.uint32), pair.cpu.w[k].view(np.uint32)), f"replay {i} key {k}"
        finally:
            pair.close()
