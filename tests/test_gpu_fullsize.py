"""Full-size GPU checks in the launch configuration the benchmark times.

The oracle cannot sweep 2^27..2^32 configurations in test time, so each
workload is checked by (i) the validity-mask count against the analytic count,
(ii) oracle predictions on sampled indices (random, range boundaries, and every
index the GPU returned), and (iii) the selection stage in full: the GPU top-k
must equal, bit for bit, the k smallest (value, index) pairs of the GPU's own
predict_all output (same kernels, same arithmetic), computed with torch ops."""
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


def exact_topk_of(pred, mask, base, k):
    """k smallest (value, index) pairs of a device prediction array (ties by index)."""
    masked = torch.where(mask.bool(), pred, torch.full_like(pred, float("inf")))
    kk = min(k, int(mask.sum().item()))
    if kk == 0:
        return np.zeros(0, np.float32), np.zeros(0, np.uint64)
    v = torch.topk(masked, kk, largest=False, sorted=True).values
    vk = v[-1]
    lt = torch.nonzero(masked < vk).flatten()
    eq = torch.nonzero((masked == vk) & mask.bool()).flatten()          # ascending
    idx = torch.cat([lt, eq[: kk - lt.numel()]])
    vals = masked[idx].cpu().numpy()
    idx = idx.cpu().numpy().astype(np.uint64) + np.uint64(base)
    order = np.lexsort((idx, vals))
    return vals[order], idx[order]


def merge_exact(parts, k):
    vals = np.concatenate([p[0] for p in parts])
    idx = np.concatenate([p[1] for p in parts])
    order = np.lexsort((idx, vals))[:k]
    return vals[order], idx[order]


def check_sampled_predictions(w, sw, n_windows, seed, returned_idx, window=4096):
    """GPU predictions on random windows of the space (plus its two ends) against
    the oracle, and the oracle's value for every configuration the GPU returned."""
    sp, m = w.space, w.model
    n = sp.n_configs
    st = wl.Stream(seed)
    begins = [0, n - window] + [int(v) for v in st.integers(n_windows, n - window)]
    worst_all, n_valid = 0.0, 0
    for begin in begins:
        pred, mask = sw.predict_all(begin, window)
        torch.cuda.synchronize()
        oy, ov, _ = oracle.predict_range(sp, m, begin, window, threads=THREADS)
        assert np.array_equal(mask.cpu().numpy(), ov)
        worst, _ = parity.check_predictions(pred.cpu().numpy(), oy, ov)
        worst_all = max(worst_all, worst)
        n_valid += int(ov.sum())
    say(f"  {w.name}: {len(begins)} windows of {window}, {n_valid} valid predictions checked, "
        f"worst {worst_all:.3f} x tol")
    assert n_valid > 0
    ry, rv = oracle.predict_indices(sp, m, returned_idx, threads=THREADS)
    assert rv.all(), "an invalid configuration was returned"
    return ry.astype(np.float64)


def test_large_2_27_topk_full():
    from paper_1506_00842_amd.api import Sweep
    w = wl.large()
    sp = w.space
    n = sp.n_configs
    sw = Sweep(sp, w.model, w.k)
    sw.topk(0, n)                                   # exactly what bench.py times
    torch.cuda.synchronize()
    gv, gi = sw.topk_host()
    assert len(gi) == w.k
    pred, mask = sw.predict_all(0, n)
    torch.cuda.synchronize()
    assert int(mask.sum().item()) == w.n_valid == 63_700_992
    assert bool(torch.all(torch.isposinf(pred[~mask.bool()])))
    ev, ei = exact_topk_of(pred, mask, 0, w.k)
    assert np.array_equal(gi, ei) and np.array_equal(gv, ev)
    ry = check_sampled_predictions(w, sw, 64, 11, gi)
    S = parity.scale_of(ry)
    assert np.all(np.abs(gv.astype(np.float64) - ry) <= parity.TOL_FP32 * np.maximum(np.abs(ry), S))
    # oracle top-k restricted to the 2^15-blocks that hold the GPU's winners plus
    # random blocks must not contain anything clearly better than the GPU's k-th value
    blocks = np.unique(gi // np.uint64(1 << 15))[:6]
    for b in blocks:
        oy, ov, _ = oracle.predict_range(sp, w.model, int(b) << 15, 1 << 15, threads=THREADS)
        band = parity.TOL_FP32 * max(abs(float(gv[-1])), S)
        better = np.nonzero(ov.astype(bool) & (oy.astype(np.float64) < float(gv[-1]) - band))[0] + (int(b) << 15)
        assert len(np.setdiff1d(better.astype(np.uint64), gi)) == 0


def test_large_2_26_as_written_and_unconstrained():
    from paper_1506_00842_amd.api import Sweep
    w = wl.large_as_written()
    n = w.space.n_configs
    sw = Sweep(w.space, w.model, w.k)
    sw.topk(0, n)
    pred, mask = sw.predict_all(0, n)
    torch.cuda.synchronize()
    assert int(mask.sum().item()) == w.n_valid == 31_850_496
    gv, gi = sw.topk_host()
    ev, ei = exact_topk_of(pred, mask, 0, w.k)
    assert np.array_equal(gi, ei) and np.array_equal(gv, ev)
    # no rules: the paper's unmasked sweep; every configuration is evaluated
    wu = wl.Workload("large-unconstrained", wl.large().space.without_constraints(), wl.large().model, 1000)
    n = wu.space.n_configs
    sw = Sweep(wu.space, wu.model, wu.k)
    sw.topk(0, n)
    pred, mask = sw.predict_all(0, n)
    torch.cuda.synchronize()
    assert int(mask.sum().item()) == n
    gv, gi = sw.topk_host()
    ev, ei = exact_topk_of(pred, mask, 0, wu.k)
    assert np.array_equal(gi, ei) and np.array_equal(gv, ev)
    check_sampled_predictions(wu, sw, 24, 5, gi)


def test_wide_2_27_topk_full():
    from paper_1506_00842_amd.api import Sweep
    w = wl.wide()
    n = w.space.n_configs
    sw = Sweep(w.space, w.model, w.k)
    sw.topk(0, n)
    torch.cuda.synchronize()
    gv, gi = sw.topk_host()
    pred, mask = sw.predict_all(0, n)
    torch.cuda.synchronize()
    assert int(mask.sum().item()) == w.n_valid
    ev, ei = exact_topk_of(pred, mask, 0, w.k)
    assert np.array_equal(gi, ei) and np.array_equal(gv, ev)
    ry = check_sampled_predictions(w, sw, 24, 12, gi)
    S = parity.scale_of(ry)
    assert np.all(np.abs(gv.astype(np.float64) - ry) <= parity.TOL_FP32 * np.maximum(np.abs(ry), S))


def test_streamed_2_32_running_topk():
    from paper_1506_00842_amd.api import Sweep
    w = wl.streamed()
    sp = w.space
    n = sp.n_configs
    chunk = w.chunk
    sw = Sweep(sp, w.model, w.k)
    for c, b in enumerate(range(0, n, chunk)):      # exactly what bench.py times
        sw.topk(b, chunk, merge=c > 0)
    torch.cuda.synchronize()
    gv, gi = sw.topk_host()
    assert len(gi) == w.k == 4096
    say("  streamed sweep done; checking the selection chunk by chunk")
    pred = torch.empty(chunk, dtype=torch.float32, device="cuda")
    mask = torch.empty(chunk, dtype=torch.uint8, device="cuda")
    parts = []
    n_valid = 0
    for b in range(0, n, chunk):
        sw.predict_all(b, chunk, out=pred, mask=mask)
        torch.cuda.synchronize()
        n_valid += int(mask.sum().item())
        parts.append(exact_topk_of(pred, mask, b, w.k))
        say(f"    chunk at {b}: valid so far {n_valid}")
    assert n_valid == w.n_valid == 3_011_788_800
    ev, ei = merge_exact(parts, w.k)
    assert np.array_equal(gi, ei) and np.array_equal(gv, ev)
    ry = check_sampled_predictions(w, sw, 48, 13, gi)
    S = parity.scale_of(ry)
    assert np.all(np.abs(gv.astype(np.float64) - ry) <= parity.TOL_FP32 * np.maximum(np.abs(ry), S))
    # a different chunk order gives the same running result
    sw2 = Sweep(sp, w.model, w.k)
    order = [7, 0, 15, 3, 1, 2, 4, 5, 6, 8, 9, 10, 11, 12, 13, 14]
    for c, j in enumerate(order):
        sw2.topk(j * chunk, chunk, merge=c > 0)
    torch.cuda.synchronize()
    v2, i2 = sw2.topk_host()
    assert np.array_equal(i2, gi) and np.array_equal(v2, gv)


@pytest.mark.parametrize("net", ["split16", "bf16"])
def test_large_2_27_other_nets_full(net):
    """The 2^27 sweep with the 16-bit matrix-core networks: selection exact against the
    path's own predictions, predictions against the oracle at the net's tolerance."""
    import paper_1506_00842_amd as T
    from paper_1506_00842_amd.api import Sweep
    kw, tol = {"split16": (dict(algo=T.TUNER_ALGO_SPLIT16), parity.TOL_FP32),
               "bf16": (dict(precision=T.TUNER_BF16_MFMA), 1e-2)}[net]
    w = wl.large()
    n = w.space.n_configs
    sw = Sweep(w.space, w.model, w.k, **kw)
    sw.topk(0, n)
    torch.cuda.synchronize()
    gv, gi = sw.topk_host()
    pred, mask = sw.predict_all(0, n)
    torch.cuda.synchronize()
    assert int(mask.sum().item()) == w.n_valid
    ev, ei = exact_topk_of(pred, mask, 0, w.k)
    assert np.array_equal(gi, ei) and np.array_equal(gv, ev)
    st = wl.Stream(21)
    worst_all = 0.0
    for begin in [0, n - 4096] + [int(v) for v in st.integers(40, n - 4096)]:
        p2, m2 = sw.predict_all(begin, 4096)
        torch.cuda.synchronize()
        oy, ov, _ = oracle.predict_range(w.space, w.model, begin, 4096, threads=THREADS)
        assert np.array_equal(m2.cpu().numpy(), ov)
        worst, _ = parity.check_predictions(p2.cpu().numpy(), oy, ov, tol=tol)
        worst_all = max(worst_all, worst)
    ry, rv = oracle.predict_indices(w.space, w.model, gi, threads=THREADS)
    assert rv.all()
    S = parity.scale_of(ry)
    assert np.all(np.abs(gv.astype(np.float64) - ry) <= tol * np.maximum(np.abs(ry), S))
    say(f"  {net}: worst {worst_all:.3f} x tol({tol:g})")
