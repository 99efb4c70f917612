"""The list push for callers that cannot allocate (-m gpu): kv_push_list_noalloc against kv_push_list.

Two stores of different sizes share the GPU's one static pointer table.  Every call of the allocation-free entry
point is compared bit for bit with the ordinary list push of a twin store fed the same buffers (and with the
oracle): a large call, then a smaller one, then the large one again, so rows left behind by one call sit next to
the rows the next call writes.  Collected last on purpose."""
from __future__ import annotations

import numpy as np
import pytest

from tests.gpu_harness import Pair, same_bits_or_both_nan, first_mismatch

pytestmark = pytest.mark.gpu

KV_ERR_ARG = -1
KV_ERR_STATE = -3
BIG = dict(numel=[70000, 5, 0, 300, 1 << 20, 1, 2049, 1024, 33, 4097, 260000, 64], W=8, bucket=64 << 10)
SMALL = dict(numel=[1000, 3, 20000], W=3, bucket=4 << 10)


def _rng(*seed):
    return np.random.Generator(np.random.SFC64([1802, *seed]))


def _grads(spec, tag, dtype):
    dt = np.float32 if dtype == "f32" else np.float16
    return [[(_rng(tag, k, r).standard_normal(n) * 0.01).astype(dt) for r in range(spec["W"])]
            for k, n in enumerate(spec["numel"])]


class Twin:
    """A store driven through kv_push_list_noalloc, a store driven through kv_push_list, and the oracle."""

    def __init__(self, spec, dtype, seed):
        import paper_1802_06949_amd as kv
        self.spec = spec
        self.dtype = dtype
        self.calls = 0
        self.pair = Pair(spec["numel"], spec["W"], dtype, spec["bucket"], lr=0.1, momentum=0.9, wd=1e-4, keep_sum=True)
        self.ref = kv.KVStore(spec["numel"], spec["W"], dtype, spec["bucket"], lr=0.1, momentum=0.9, wd=1e-4, keep_sum=True)
        w0 = [_rng(seed, k).standard_normal(n).astype(np.float32) for k, n in enumerate(spec["numel"])]
        self.pair.set_weights(w0)
        import torch
        for k, w in enumerate(w0):
            if w.size:
                self.ref.set_weights(k, torch.from_numpy(w).cuda())
        self.ref.wait()

    def step(self, tag, keys=None):
        import torch
        K = len(self.spec["numel"])
        g = _grads(self.spec, tag, self.dtype)
        dev = self.pair.upload(g)                        # fresh buffers: no cached table has ever held them
        keys = list(range(K)) if keys is None else keys
        pl = self.pair.gpu.make_push_list(keys, [dev[k] for k in keys])
        free_before = torch.cuda.mem_get_info()[0]
        self.pair.gpu.push_list_noalloc(pl)
        if self.calls > 0:           # the first launch of a kernel in a process makes the runtime load its code
            assert torch.cuda.mem_get_info()[0] == free_before, "device memory changed hands during the call"
        self.calls += 1
        self.ref.push_list(self.ref.make_push_list(keys, [dev[k] for k in keys]))
        return g

    def finish(self, g, label):
        import torch
        self.pair.gpu.wait()
        self.ref.wait()
        self.pair.cpu.step(g)
        self.pair.compare(label + " vs oracle")
        for k, n in enumerate(self.spec["numel"]):
            for what, fn in (("w", self.ref.pull), ("m", self.ref.pull_momentum), ("s", self.ref.pull_grad)):
                out = torch.empty(n, dtype=torch.float32, device="cuda")
                fn(k, out)
                self.ref.wait()
                got = self.pair.fetch(what, k)
                assert same_bits_or_both_nan(got, out.cpu().numpy()), \
                    f"{label} key {k} {what} vs kv_push_list: {first_mismatch(got, out.cpu().numpy())}"

    def close(self):
        self.pair.close()
        self.ref.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_noalloc_push_matches_the_list_push_large_then_small(dtype):
    big, small = Twin(BIG, dtype, 1), Twin(SMALL, dtype, 2)
    try:
        big.finish(big.step(10), "large call")
        small.finish(small.step(11), "smaller call after the large one")
        big.finish(big.step(12), "large call again")
        # one iteration handed over in two lists (the second completes the units), on the small store
        K = len(SMALL["numel"])
        g = _grads(SMALL, 13, dtype)
        dev = small.pair.upload(g)
        for part in ([2], [1, 0]):
            small.pair.gpu.push_list_noalloc(small.pair.gpu.make_push_list(part, [dev[k] for k in part]))
            small.ref.push_list(small.ref.make_push_list(part, [dev[k] for k in part]))
        small.finish(g, "iteration pushed in two lists")
        assert K == 3
    finally:
        big.close()
        small.close()


def test_noalloc_push_rejects_what_does_not_fit_and_other_schedules():
    import torch
    import paper_1802_06949_amd as kv
    numel = [1] * 300
    st = kv.KVStore(numel, 256, "f32", 1 << 10, lr=0.1)          # 300 x 256 = 76 800 pointers > 65 536
    try:
        g = torch.zeros(1, device="cuda")
        pl = st.make_push_list([0], [[g] * 256])
        with pytest.raises(kv.KVError) as e:
            st.push_list_noalloc(pl)
        assert e.value.status == KV_ERR_ARG and "65536" in str(e.value)
        st.wait()                                                  # nothing was marked
    finally:
        st.close()
    st = kv.KVStore([100, 200], 2, "f32", 1 << 10, lr=0.1)
    try:
        st.set_schedule(kv.KV_SCHED_FUNNEL)
        g = [torch.zeros(200, device="cuda") for _ in range(2)]
        with pytest.raises(kv.KVError) as e:
            st.push_list_noalloc(st.make_push_list([1], [g]))
        assert e.value.status == KV_ERR_STATE
    finally:
        st.close()


def test_noalloc_push_is_captured_without_an_earlier_push_of_the_buffers():
    import torch
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        spec = SMALL
        pair = Pair(spec["numel"], spec["W"], "f32", spec["bucket"], lr=0.1, momentum=0.9, wd=1e-4, keep_sum=True,
                    stream=s.cuda_stream)
        try:
            pair.set_weights([_rng(5, k).standard_normal(n).astype(np.float32) for k, n in enumerate(spec["numel"])])
            K = len(spec["numel"])
            gA = _grads(spec, 20, "f32")
            dA = pair.upload(gA)                               # never pushed before the capture
            pl = pair.gpu.make_push_list(list(range(K)), dA)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=s):
                pair.gpu.push_list_noalloc(pl)
            s.synchronize()
            pair.compare("a capture runs nothing")
            for i in range(3):
                graph.replay()
                pair.cpu.step(gA)
                pair.gpu.wait()
                pair.compare(f"replay {i}")
                gB = _grads(spec, 30 + i, "f32")               # eager allocation-free step in between: other rows
                dB = pair.upload(gB)
                pair.gpu.push_list_noalloc(pair.gpu.make_push_list(list(range(K)), dB))
                pair.gpu.wait()
                pair.cpu.step(gB)
                pair.compare(f"eager step after replay {i}")
        finally:
            pair.close()
