"""The allocation-free entry point (tuner_predict_topk_static: the sweep's scratch lives in a
device array inside the library) against tuner_predict_topk with a caller workspace: same
kernels on the same inputs, so values, indices and n_found must agree bit for bit.  Calls
go through the C ABI; two calls in a row share the one array, the second with a smaller
input, and the array is left as the previous call wrote it."""
import os

import numpy as np
import pytest

import oracle
import parity
import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)


def say(*a):
    print(*a, flush=True)


class StaticTopk:
    """Outputs for tuner_predict_topk_static next to a Sweep that owns a workspace."""

    def __init__(self, w, k=None, **kw):
        from paper_1506_00842_amd.api import Sweep
        self.k = w.k if k is None else k
        self.ref = Sweep(w.space, w.model, self.k, **kw)
        dev = self.ref.device
        self.values = torch.full((self.k,), -7.0, dtype=torch.float32, device=dev)
        self.indices = torch.full((self.k,), 7, dtype=torch.int32, device=dev)
        self.n_found = torch.full((1,), -7, dtype=torch.int32, device=dev)

    def topk(self, begin, count, merge=False):
        import paper_1506_00842_amd as T
        T.tuner_predict_topk_static(self.ref.space, self.ref.model, begin, count, self.k, 1 if merge else 0,
                                    self.values, self.indices, self.n_found)

    def host(self):
        n = int(self.n_found.item())
        return (self.values[:n].cpu().numpy(),
                self.indices[:n].cpu().numpy().view(np.uint32).astype(np.uint64))

    def same_as_reference(self):
        torch.cuda.synchronize()
        assert torch.equal(self.n_found, self.ref.n_found)
        # whole buffers: the tail past n_found is (+inf, 0xFFFFFFFF) in both
        assert torch.equal(self.values.view(torch.int32), self.ref.values.view(torch.int32))
        assert torch.equal(self.indices, self.ref.indices)


def test_static_scratch_two_calls_in_a_row_second_smaller():
    # first call: a long constrained range of the 2^27 space (live-chunk list, work queue,
    # candidate pools all in the scratch), k = 1000
    w1 = wl.large()
    begin, count = (5 << 20) + 12345, (1 << 23) + 4321
    s1 = StaticTopk(w1)
    say("static call 1:", w1.name, begin, count, "k", s1.k)
    s1.topk(begin, count)
    s1.ref.topk(begin, count)
    s1.same_as_reference()
    gv, gi = s1.host()
    assert len(gi) == 1000
    ry, rv = oracle.predict_indices(w1.space, w1.model, gi, threads=THREADS)
    assert rv.all()
    S = parity.scale_of(ry)
    assert np.all(np.abs(gv.astype(np.float64) - ry) <= parity.TOL_FP32 * np.maximum(np.abs(ry), S))

    # second call, right behind it, on a smaller problem: another space, another model, a
    # smaller k; the scratch still holds the first call's header, tables, weights and lists
    w2 = wl.conv_shaped()
    n2 = w2.space.n_configs
    s2 = StaticTopk(w2)
    say("static call 2:", w2.name, 0, n2, "k", s2.k)
    s2.topk(0, n2)
    s2.ref.topk(0, n2)
    s2.same_as_reference()
    oy, ov, _ = oracle.predict_range(w2.space, w2.model, 0, n2, threads=THREADS)
    gv, gi = s2.host()
    parity.check_topk(gv, gi, oy, ov, 0, w2.k)

    # a third, smaller still and ragged, merging with the result of a fourth
    s2.topk(1000, 70001)
    s2.ref.topk(1000, 70001)
    s2.same_as_reference()
    s2.topk(200000, 33, merge=True)
    s2.ref.topk(200000, 33, merge=True)
    s2.same_as_reference()

    # and the first problem again: nothing of the smaller calls leaks into it
    s1.topk(begin, count)
    s1.same_as_reference()


def test_static_scratch_chunked_running_result_and_other_networks():
    import paper_1506_00842_amd as T
    w = wl.paper_raycasting()
    n = w.space.n_configs
    for kw in (dict(), dict(precision=T.TUNER_BF16_MFMA), dict(algo=T.TUNER_ALGO_SPLIT16), dict(algo=T.TUNER_ALGO_VALU)):
        s = StaticTopk(w, **kw)
        cuts = [0, 300001, 300002, n]
        for j, (b, e) in enumerate(zip(cuts[:-1], cuts[1:])):
            s.topk(b, e - b, merge=j > 0)
            s.ref.topk(b, e - b, merge=j > 0)
        s.same_as_reference()
        # empty range: a fresh call gives an empty result
        s.topk(5, 0)
        s.ref.topk(5, 0)
        s.same_as_reference()
        assert int(s.n_found.item()) == 0


def test_static_scratch_call_records_no_timing_events():
    """Timing a call means creating HIP events; the call that allocates nothing creates none,
    also while timing is switched on (the plain call beside it records one pair)."""
    import paper_1506_00842_amd as T
    w = wl.conv_shaped()
    s = StaticTopk(w)
    T.tuner_profile_enable(True)
    try:
        T.tuner_profile_read()
        s.topk(0, w.space.n_configs)
        torch.cuda.synchronize()
        assert T.tuner_profile_pending() == 0
        s.ref.topk(0, w.space.n_configs)
        torch.cuda.synchronize()
        assert T.tuner_profile_pending() == 1
        s.same_as_reference()
    finally:
        T.tuner_profile_enable(False)
    assert T.tuner_profile_pending() == 0


def test_static_scratch_refuses_what_does_not_fit():
    import paper_1506_00842_amd as T
    w = wl.large()
    s = StaticTopk(w, k=16384)          # pools for k = 16384 need 128 MiB
    assert T.tuner_workspace_bytes(s.ref.space, s.ref.model, 16384) > T.TUNER_STATIC_SCRATCH_BYTES
    with pytest.raises(T.TunerError) as e:
        s.topk(0, 1 << 20)
    assert e.value.code == T.TUNER_ETOOLARGE
    assert "static" in str(e.value)
    torch.cuda.synchronize()
    # outputs untouched
    assert bool(torch.all(s.values == -7.0)) and bool(torch.all(s.indices == 7)) and int(s.n_found.item()) == -7
    # the streamed configuration (k = 4096, 2^32 configurations) fits
    ws = wl.streamed()
    s5 = StaticTopk(ws)
    assert T.tuner_workspace_bytes(s5.ref.space, s5.ref.model, ws.k) <= T.TUNER_STATIC_SCRATCH_BYTES
    s5.topk((1 << 32) - (1 << 22), 1 << 22)
    s5.ref.topk((1 << 32) - (1 << 22), 1 << 22)
    s5.same_as_reference()
