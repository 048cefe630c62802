"""Full-size GPU checks in the launch configuration the benchmark times.

The oracle cannot sweep 2^27..2^32 configurations in test time, so each
workload is checked by (i) the validity-mask count against the analytic count,
(ii) oracle predictions on windows of the long sweep's own output (random places and
the two ends) and at every index the GPU returned, and (iii) the selection stage in full: the GPU top-k
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


def check_windows_of_a_long_sweep(w, pred, mask, base, n_windows, seed, tol=parity.TOL_FP32, window=4096):
    """Windows of a long sweep's own output (device tensors over [base, base + len)) against
    the oracle: what is checked is what the full-size launch wrote (work queue, live-chunk
    list, full chunks), not a fresh short call.  The two ends of the range and random places."""
    sp, m = w.space, w.model
    n = pred.numel()
    st = wl.Stream(seed)
    offsets = [0, n - window] + [int(v) for v in st.integers(n_windows, n - window)]
    worst_all, n_valid = 0.0, 0
    for t0 in offsets:
        oy, ov, _ = oracle.predict_range(sp, m, base + t0, window, threads=THREADS)
        assert np.array_equal(mask[t0:t0 + window].cpu().numpy(), ov)
        worst, _ = parity.check_predictions(pred[t0:t0 + window].cpu().numpy(), oy, ov, tol=tol)
        worst_all = max(worst_all, worst)
        n_valid += int(ov.sum())
    say(f"  {w.name}: {len(offsets)} windows of {window} of the long sweep's output, {n_valid} valid "
        f"predictions checked, worst {worst_all:.3f} x tol({tol:g})")
    assert n_valid > 0


def oracle_at_returned(w, gv, gi, tol=parity.TOL_FP32):
    """The oracle's value at every configuration the GPU returned: all valid, values within tol."""
    ry, rv = oracle.predict_indices(w.space, w.model, gi, threads=THREADS)
    assert rv.all(), "an invalid configuration was returned"
    ry = ry.astype(np.float64)
    S = parity.scale_of(ry)
    assert np.all(np.abs(gv.astype(np.float64) - ry) <= tol * np.maximum(np.abs(ry), S))
    return ry, S


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
    check_windows_of_a_long_sweep(w, pred, mask, 0, 64, 11)
    ry, S = oracle_at_returned(w, gv, gi)
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
    check_windows_of_a_long_sweep(wu, pred, mask, 0, 24, 5)
    oracle_at_returned(wu, gv, gi)


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
    check_windows_of_a_long_sweep(w, pred, mask, 0, 24, 12)
    oracle_at_returned(w, gv, gi)


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
        check_windows_of_a_long_sweep(w, pred, mask, b, 2, 13 + b // chunk)
        say(f"    chunk at {b}: valid so far {n_valid}")
    assert n_valid == w.n_valid == 3_011_788_800
    ev, ei = merge_exact(parts, w.k)
    assert np.array_equal(gi, ei) and np.array_equal(gv, ev)
    oracle_at_returned(w, gv, gi)
    # a different chunk order gives the same running result
    sw2 = Sweep(sp, w.model, w.k)
    order = [7, 0, 15, 3, 1, 2, 4, 5, 6, 8, 9, 10, 11, 12, 13, 14]
    for c, j in enumerate(order):
        sw2.topk(j * chunk, chunk, merge=c > 0)
    torch.cuda.synchronize()
    v2, i2 = sw2.topk_host()
    assert np.array_equal(i2, gi) and np.array_equal(v2, gv)


@pytest.mark.parametrize("maker,net", [(wl.large, "split16"), (wl.large, "bf16"), (wl.large, "valu"),
                                       (wl.wide, "bf16"), (wl.wide, "split16"), (wl.wide, "valu")])
def test_2_27_other_nets_full(maker, net):
    """The 2^27 sweeps (64-wide and 128-wide ensembles) with the other network evaluations, in
    the launch configuration the benchmark times: mask count, selection exact against the
    path's own predictions, windows of the long sweep's output and every returned
    configuration against the oracle at the net's tolerance (1e-2 for bf16 operands)."""
    import paper_1506_00842_amd as T
    from paper_1506_00842_amd.api import Sweep
    kw, tol = {"split16": (dict(algo=T.TUNER_ALGO_SPLIT16), parity.TOL_FP32),
               "valu": (dict(algo=T.TUNER_ALGO_VALU), parity.TOL_FP32),
               "bf16": (dict(precision=T.TUNER_BF16_MFMA), 1e-2)}[net]
    w = maker()
    n = w.space.n_configs
    sw = Sweep(w.space, w.model, w.k, **kw)
    plan = T.tuner_sweep_plan(sw.space, sw.model, 0, n, w.k)
    assert plan["tiles_per_wave"] == plan["variant_tiles_per_wave"] and plan["dynamic_queue"] == 1
    say(f"  {w.name} {net}: {plan}")
    sw.topk(0, n)
    torch.cuda.synchronize()
    gv, gi = sw.topk_host()
    pred, mask = sw.predict_all(0, n)
    torch.cuda.synchronize()
    assert int(mask.sum().item()) == w.n_valid
    assert bool(torch.all(torch.isposinf(pred[~mask.bool()])))
    ev, ei = exact_topk_of(pred, mask, 0, w.k)
    assert np.array_equal(gi, ei) and np.array_equal(gv, ev)
    check_windows_of_a_long_sweep(w, pred, mask, 0, 40 if maker is wl.large else 24, 21, tol=tol)
    oracle_at_returned(w, gv, gi, tol=tol)


@pytest.mark.slow
def test_large_2_27_full_space_against_the_oracle():
    """Every one of the 2^27 predictions of the benchmarked launch against the oracle (all
    host threads, about a minute): mask bit for bit, predictions at the fp32 tolerance, and
    the returned top-1000 against the oracle's own full-space selection by the band rule."""
    from paper_1506_00842_amd.api import Sweep
    w = wl.large()
    sp = w.space
    n = sp.n_configs
    sw = Sweep(sp, w.model, w.k)
    sw.topk(0, n)
    pred, mask = sw.predict_all(0, n)
    torch.cuda.synchronize()
    gv, gi = sw.topk_host()
    g_pred = pred.cpu().numpy()
    g_mask = mask.cpu().numpy()
    del pred, mask
    o_pred = np.empty(n, np.float32)
    o_mask = np.empty(n, np.uint8)
    piece = 1 << 24
    worst_all = 0.0
    for b in range(0, n, piece):
        oy, ov, _ = oracle.predict_range(sp, w.model, b, piece, threads=THREADS)
        o_pred[b:b + piece] = oy
        o_mask[b:b + piece] = ov
        assert np.array_equal(g_mask[b:b + piece], ov)
        worst, _ = parity.check_predictions(g_pred[b:b + piece], oy, ov)
        worst_all = max(worst_all, worst)
        say(f"    oracle piece at {b}: worst so far {worst_all:.3f} x tol")
    assert int(o_mask.sum()) == w.n_valid
    parity.check_topk(gv, gi, o_pred, o_mask, 0, w.k)
    # the oracle's own selection, for the record: how many of its 1000 the GPU returned
    _, oi = oracle.select_topk(o_pred, o_mask, 0, w.k)
    say(f"  full space: worst {worst_all:.3f} x tol; {len(np.intersect1d(oi, gi))} of {w.k} indices in common "
        "with the oracle's selection (the rest lie within the band around the k-th value)")


@pytest.mark.parametrize("radices,begin,count", [
    ([8, 8, 8, 8, 4, 4, 4, 4, 4, 2, 2, 2, 2, 2], 12345, (1 << 24) + 777),          # powers of two, ragged range
    ([8, 5, 8, 3, 4, 4, 3, 4, 4, 2, 2, 3, 2, 2], 1000003, (1 << 24) + 12345),      # multiply-shift decoder
])
def test_long_range_with_rules_on_low_parameters(radices, begin, count):
    """A long sweep visits a list of live chunks made from each chunk's two end points.
    Here the range starts off any chunk boundary and the rules touch high, middle and
    low parameters, so chunks are wholly invalid, wholly valid or mixed: the mask of the
    whole range against the oracle's (integer work only), the top-k against the exact
    selection from the GPU's own predictions, and sampled predictions against the oracle."""
    from paper_1506_00842_amd.api import Sweep
    values = [[float(1 << j) for j in range(r)] if r > 2 else [0.0, 1.0] for r in radices]
    scales = [wl.SCALE_LOG2 if r > 2 else wl.SCALE_LINEAR for r in radices]
    total = sum(radices)
    off = np.concatenate([[0], np.cumsum(radices)])[:-1]
    terms = np.zeros((4, total), np.int32)
    for p in (0, 1):                                   # high: d0 + d1 <= 9
        terms[0, off[p]:off[p] + radices[p]] = np.arange(radices[p])
    terms[1, off[2]:off[2] + radices[2]] = np.arange(radices[2])      # high: d2 <= d3 + 4
    terms[1, off[3]:off[3] + radices[3]] = -np.arange(radices[3])
    for p in (6, 7):                                   # middle (strides around one chunk): d6 + d7 <= 4
        terms[2, off[p]:off[p] + radices[p]] = np.arange(radices[p])
    for p in (10, 11, 13):                             # low (inside a tile): d10 + d11 + d13 <= 2
        terms[3, off[p]:off[p] + radices[p]] = np.arange(radices[p])
    sp = wl.Space("mixed-chunks", values, scales, terms, np.array([9, 4, 4, 2], np.int64))
    assert begin + count <= sp.n_configs
    w = wl.Workload("mixed-chunks", sp, wl.make_model([14, 64, 64, 1], 2, 77), 500)
    sw = Sweep(sp, w.model, w.k)
    sw.topk(begin, count)
    pred, mask = sw.predict_all(begin, count)
    torch.cuda.synchronize()
    _, ov, _ = oracle.predict_range(sp, None, begin, count, threads=THREADS, want_yhat=False)
    gm = mask.cpu().numpy()
    assert np.array_equal(gm, ov)
    say(f"  {int(ov.sum())} of {count} valid")
    assert 0.05 < ov.mean() < 0.95
    assert bool(torch.all(torch.isposinf(pred[~mask.bool()])))
    gv, gi = sw.topk_host()
    ev, ei = exact_topk_of(pred, mask, begin, w.k)
    assert np.array_equal(gi, ei) and np.array_equal(gv, ev)
    # values: windows of the long run's own output against the oracle
    st = wl.Stream(5)
    for t0 in [0, count - 3000] + [int(v) for v in st.integers(6, count - 3000)]:
        oy, ov2, _ = oracle.predict_range(sp, w.model, begin + t0, 3000, threads=THREADS)
        assert np.array_equal(gm[t0:t0 + 3000], ov2)
        parity.check_predictions(pred[t0:t0 + 3000].cpu().numpy(), oy, ov2)
    ry, rv = oracle.predict_indices(sp, w.model, gi, threads=THREADS)
    assert rv.all()
