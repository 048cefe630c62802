"""GPU parity tests: the HIP path (through the C ABI) against the CPU oracle on
the same seeded inputs.  Decoded digits, features and the validity mask are
compared bit for bit; predictions within 1e-5 (scaled, see parity.py); top-k by
the band rule.  Run with -m gpu on an MI355X."""
import os

import numpy as np
import pytest

import oracle
import parity
import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)


def sweep_for(w, k=None, **kw):
    from paper_1506_00842_amd.api import Sweep
    return Sweep(w.space, w.model, w.k if k is None else k, **kw)


def say(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------ decode ---
DECODE_CASES = [
    (wl.tiny, 0, 256), (wl.conv_shaped, 0, 393216), (wl.paper_raycasting, 655360 - 70001, 70001),
    (wl.paper_stereo, 1234567, 99999), (wl.large, (1 << 27) - 100003, 100003),
    (wl.streamed, (1 << 32) - 65539, 65539), (wl.streamed, (1 << 31) - 777, 5000),
    (lambda: wl.random_small(5), 0, None), (lambda: wl.many_params(25, [8], 1, 3), 188743680 - 50000, 50000),
]


@pytest.mark.parametrize("maker,begin,count", DECODE_CASES)
def test_decode_features_mask_bit_exact(maker, begin, count):
    w = maker()
    sp = w.space
    count = sp.n_configs if count is None else count
    say("decode", sp.name, begin, count)
    sw = sweep_for(w, k=0)
    d, f, v = sw.decode(begin, count)
    torch.cuda.synchronize()
    _, ov, od = oracle.predict_range(sp, None, begin, count, threads=THREADS, want_yhat=False, want_digits=True)
    assert np.array_equal(d.cpu().numpy(), od)
    assert np.array_equal(v.cpu().numpy(), ov)
    lut = oracle.feature_lut(sp)
    of = np.stack([lut[sp.offsets[p] + od[:, p]] for p in range(sp.n_params)], axis=1)
    assert np.array_equal(f.cpu().numpy(), of)


# ------------------------------------------------------------ predict_all ----
def _check_range(w, begin, count, sw=None):
    sp, m = w.space, w.model
    sw = sw or sweep_for(w, k=0)
    pred, mask = sw.predict_all(begin, count)
    torch.cuda.synchronize()
    oy, ov, _ = oracle.predict_range(sp, m, begin, count, threads=THREADS)
    assert np.array_equal(mask.cpu().numpy(), ov)
    worst, rel = parity.check_predictions(pred.cpu().numpy(), oy, ov)
    say(f"  {w.name} [{begin}, +{count}): worst {worst:.3f} x tol, pure-relative worst {rel:.2e}")


def test_predict_all_tiny_and_conv_full():
    for maker in (wl.tiny, wl.conv_shaped):
        w = maker()
        _check_range(w, 0, w.space.n_configs)


@pytest.mark.parametrize("maker", [wl.paper_convolution, wl.paper_raycasting, wl.paper_stereo])
def test_predict_all_paper_spaces_full(maker):
    w = maker()
    _check_range(w, 0, w.space.n_configs)


SHAPES = [  # (n_params, hidden widths, members): every kernel family and padding
    (3, [5], 1), (7, [30], 11), (7, [33], 2), (9, [64], 3), (12, [100], 2), (15, [128], 2),
    (16, [20], 3), (23, [32], 2), (24, [64], 2), (31, [17], 2),
    (5, [7, 7], 2), (10, [32, 32], 3), (14, [40, 20], 3), (14, [20, 60], 2), (14, [64, 64], 4),
    (14, [128, 128], 3), (14, [100, 70], 2), (20, [64, 64], 8), (26, [33, 31], 2), (31, [128, 100], 2),
]


@pytest.mark.parametrize("P,hidden,E", SHAPES)
def test_predict_all_model_shapes(P, hidden, E):
    w = wl.many_params(P, hidden, E, seed=100 + P + len(hidden))
    n = w.space.n_configs
    count = min(n, 20011)                      # ragged: not a multiple of the tile or chunk
    begin = min((n // 3) | 1, n - count)
    _check_range(w, begin, count)
    wp = wl.many_params(P, hidden, E, seed=7, pow2=True)
    n = wp.space.n_configs
    count = min(n, 9001)
    _check_range(wp, n - count, count)


# How many configurations the fastest parameters span decides how the fp32 matrix network
# evaluates layer 1: (4, 3, 3) = 36 -> high share once per tile, matrix steps over the rest;
# (2, 4, 4), (8, 4) and (32,) = 32 -> the rest from the per-member table.
@pytest.mark.parametrize("tail", [(4, 3, 3), (2, 4, 4), (8, 4), (32,), (3, 16)])
@pytest.mark.parametrize("P,hidden,E", [(7, [30], 11), (9, [64], 3), (12, [100], 2), (14, [64, 64], 4),
                                        (14, [128, 128], 1), (20, [64, 64], 8), (23, [33, 31], 2)])
def test_predict_all_layer1_shortcuts(P, hidden, E, tail):
    for pow2 in (False, True):
        w = wl.many_params(P, hidden, E, seed=300 + P + sum(tail), pow2=pow2, tail=tail)
        n = w.space.n_configs
        assert n <= 1 << 32
        count = min(n, 15013)
        begin = min((n // 5) | 1, n - count)       # odd: the first tile starts before the range
        _check_range(w, begin, count)


def test_predict_all_ragged_and_empty_ranges():
    w = wl.conv_shaped()
    sw = sweep_for(w, k=0)
    for begin, count in ((0, 1), (31, 2), (1023, 1026), (393216 - 1, 1), (5000, 4097), (77, 31)):
        _check_range(w, begin, count, sw)
    # empty range: nothing is written
    out = torch.full((8,), -1.0, device="cuda")
    sw.predict_all(100, 0, want_mask=False, out=out)
    torch.cuda.synchronize()
    assert torch.all(out == -1.0)


def test_predict_all_large_and_wide_slices():
    for maker, count in ((wl.large, 1 << 18), (wl.wide, 1 << 15), (wl.streamed, 1 << 17)):
        w = maker()
        sw = sweep_for(w, k=0)
        n = w.space.n_configs
        # slices that contain both valid and invalid blocks
        for begin in (0, (37 << 15) + 4321, n - count):
            _check_range(w, begin, count, sw)


def test_saturation_zero_weights_and_constant_net():
    w = wl.conv_shaped()
    m = w.model
    z = wl.Model(m.widths, m.n_members, np.zeros_like(m.weights))
    fpm = z.floats_per_member
    for e in range(z.n_members):
        z.weights[(e + 1) * fpm - 1] = 0.5 * (e + 1)
    wz = wl.Workload("zero", w.space, z, 25)
    sw = sweep_for(wz)
    pred, mask = sw.predict_all(0, 50000)
    sw.topk(0, w.space.n_configs)
    torch.cuda.synchronize()
    g = pred.cpu().numpy()
    ok = mask.cpu().numpy().astype(bool)
    assert np.all(g[ok] == np.float32(0.5 * 36 / 8))          # mean of the output biases
    # all predictions equal: the k smallest are the first k valid indices
    _, ov, _ = oracle.predict_range(w.space, None, 0, 5000, want_yhat=False)
    gv, gi = sw.topk_host()
    assert list(gi) == list(np.nonzero(ov)[0][:25])
    # saturated sigmoids stay finite
    big = wl.Model(m.widths, 1, np.zeros(fpm, np.float32))
    (W1, b1), (wo, bo) = big.member_layers(0)
    b1[:15] = 1e4
    b1[15:] = -1e4
    wo[:] = 1.0
    sw2 = sweep_for(wl.Workload("sat", w.space, big, 5))
    pred, mask = sw2.predict_all(0, 4096)
    torch.cuda.synchronize()
    g = pred.cpu().numpy()[mask.cpu().numpy().astype(bool)]
    assert np.all(g == 15.0)


# ------------------------------------------------- other network evaluations --
TOL_BF16 = 1e-2


def _nets():
    import paper_1506_00842_amd as T
    return {"split16": (dict(precision=T.TUNER_FP32, algo=T.TUNER_ALGO_SPLIT16), parity.TOL_FP32),
            "valu": (dict(precision=T.TUNER_FP32, algo=T.TUNER_ALGO_VALU), parity.TOL_FP32),
            "bf16": (dict(precision=T.TUNER_BF16_MFMA, algo=T.TUNER_ALGO_AUTO), TOL_BF16)}


@pytest.mark.parametrize("net", ["split16", "bf16", "valu"])
@pytest.mark.parametrize("P,hidden,E", SHAPES)
def test_other_nets_model_shapes(net, P, hidden, E):
    """Two-plane f16 split (fp32 tolerance) and bf16 operands (1e-2) on every
    kernel family and padding, ragged ranges, mixed and power-of-two radices."""
    kw, tol = _nets()[net]
    for pow2 in (False, True):
        w = wl.many_params(P, hidden, E, seed=200 + P + len(hidden), pow2=pow2)
        n = w.space.n_configs
        count = min(n, 12007)
        begin = min((n // 5) | 1, n - count)
        sw = sweep_for(w, k=0, **kw)
        pred, mask = sw.predict_all(begin, count)
        torch.cuda.synchronize()
        oy, ov, _ = oracle.predict_range(w.space, w.model, begin, count, threads=THREADS)
        assert np.array_equal(mask.cpu().numpy(), ov)
        worst, _ = parity.check_predictions(pred.cpu().numpy(), oy, ov, tol=tol)
        say(f"  {net} {w.name} {hidden}: worst {worst:.3f} x tol({tol:g})")


@pytest.mark.parametrize("net", ["split16", "bf16", "valu"])
def test_other_nets_benchmark_workloads(net):
    kw, tol = _nets()[net]
    for maker, begin, count in ((wl.tiny, 0, 256), (wl.conv_shaped, 0, 393216),
                                (wl.paper_stereo, 2359296 - 150001, 150001),
                                (wl.large, (37 << 15) + 4321, 1 << 17), (wl.wide, (37 << 15), 1 << 14),
                                (wl.streamed, (1 << 32) - (1 << 16), 1 << 16)):
        w = maker()
        sw = sweep_for(w, **kw)
        pred, mask = sw.predict_all(begin, count)
        torch.cuda.synchronize()
        oy, ov, _ = oracle.predict_range(w.space, w.model, begin, count, threads=THREADS)
        assert np.array_equal(mask.cpu().numpy(), ov)
        worst, _ = parity.check_predictions(pred.cpu().numpy(), oy, ov, tol=tol)
        # top-k of the same range under the band rule at this net's tolerance
        sw.topk(begin, count)
        torch.cuda.synchronize()
        gv, gi = sw.topk_host()
        parity.check_topk(gv, gi, oy, ov, begin, w.k, tol=tol)
        say(f"  {net} {w.name}: worst {worst:.3f} x tol({tol:g}), top-{w.k} ok")


# The 128-wide bf16 network runs with 16 waves per workgroup and two tiles per wave in a chunk
# (1024 configurations); short calls use one tile per wave.  The same range is swept in one
# call and in calls of 2^13 configurations: parity with the oracle at the bf16 tolerance, and
# the same bits both ways (what a configuration's prediction is does not depend on how a
# sweep is cut into calls or on the chunk shape).
WIDE_BF16_RANGES = [
    # (begin, count): parameter 2 has stride 2^18 and parameter 3 stride 2^15 in this space,
    # and a configuration is valid iff digit 2 <= digit 3 (and digit 0 + digit 1 <= 10): a
    # range of 2^18 from a block with digit 2 = 3 has three invalid and five valid blocks of
    # 2^15, each a run of wholly invalid or wholly valid chunks
    ((3 << 18) + 4321, (1 << 18) - 5),
    # a long range (work queue and live-chunk list, full chunks) across a change of digit 1
    # with digit 0 + digit 1 = 10 -> 11 (valid -> all invalid), ragged at both ends
    ((3 << 24) + (7 << 21) + (2 << 18) + 31, (1 << 21) + 777),
]


@pytest.mark.parametrize("begin,count", WIDE_BF16_RANGES)
def test_wide_bf16_long_ranges_against_oracle_and_short_calls(begin, count):
    import paper_1506_00842_amd as T
    w = wl.wide()
    sw = sweep_for(w, precision=T.TUNER_BF16_MFMA)
    plan = T.tuner_sweep_plan(sw.space, sw.model, begin, count, 0)
    say("wide bf16", begin, count, plan)
    assert plan["waves"] == 16 and plan["variant_tiles_per_wave"] == 2
    if count >= 1 << 21:
        assert plan["tiles_per_wave"] == 2 and plan["dynamic_queue"] == 1 and plan["live_chunk_list"] == 1
    pred, mask = sw.predict_all(begin, count)
    torch.cuda.synchronize()
    oy, ov, _ = oracle.predict_range(w.space, w.model, begin, count, threads=THREADS)
    assert np.array_equal(mask.cpu().numpy(), ov)
    assert 0.15 < ov.mean() < 0.85                     # both kinds of chunks are in the range
    worst, rel = parity.check_predictions(pred.cpu().numpy(), oy, ov, tol=TOL_BF16)
    say(f"  one call: worst {worst:.3f} x tol(1e-2), pure-relative worst {rel:.2e}")
    # the same range in pieces of 2^13 configurations: one tile per wave
    piece = 1 << 13
    assert T.tuner_sweep_plan(sw.space, sw.model, begin, piece, 0)["tiles_per_wave"] == 1
    pred2 = torch.empty_like(pred)
    mask2 = torch.empty_like(mask)
    for t0 in range(0, count, piece):
        c = min(piece, count - t0)
        sw.predict_all(begin + t0, c, out=pred2[t0:t0 + c], mask=mask2[t0:t0 + c])
    torch.cuda.synchronize()
    assert torch.equal(mask, mask2)
    assert torch.equal(pred.view(torch.int32), pred2.view(torch.int32)), "long and short calls differ in bits"
    # top-k: one call against the running result over the pieces (bit-identical), and the
    # band rule against the oracle at the bf16 tolerance
    sw.topk(begin, count)
    torch.cuda.synchronize()
    gv, gi = sw.topk_host()
    parity.check_topk(gv, gi, oy, ov, begin, w.k, tol=TOL_BF16)
    sw2 = sweep_for(w, precision=T.TUNER_BF16_MFMA)
    for j, t0 in enumerate(range(0, count, piece)):
        sw2.topk(begin + t0, min(piece, count - t0), merge=j > 0)
    torch.cuda.synchronize()
    gv2, gi2 = sw2.topk_host()
    assert np.array_equal(gi, gi2) and np.array_equal(gv, gv2)


def test_split16_saturation_and_zero_weights():
    import paper_1506_00842_amd as T
    w = wl.conv_shaped()
    m = w.model
    fpm = m.floats_per_member
    big = wl.Model(m.widths, 1, np.zeros(fpm, np.float32))
    (W1, b1), (wo, bo) = big.member_layers(0)
    b1[:15] = 1e4
    b1[15:] = -1e4
    wo[:] = 1.0
    for kw in (dict(algo=T.TUNER_ALGO_SPLIT16), dict(precision=T.TUNER_BF16_MFMA), dict(algo=T.TUNER_ALGO_VALU)):
        sw = sweep_for(wl.Workload("sat", w.space, big, 5), **kw)
        pred, mask = sw.predict_all(0, 4096)
        torch.cuda.synchronize()
        g = pred.cpu().numpy()[mask.cpu().numpy().astype(bool)]
        assert np.all(g == 15.0)


# ------------------------------------------------------------------- top-k ---
def test_topk_small_spaces_exact_and_band():
    for maker in (wl.tiny, wl.conv_shaped, lambda: wl.random_small(2), lambda: wl.random_small(4),
                  wl.paper_convolution):
        w = maker()
        sp = w.space
        n = sp.n_configs
        oy, ov, _ = oracle.predict_range(sp, w.model, 0, n, threads=THREADS)
        n_valid = int(ov.sum())
        for k in sorted({1, 2, w.k, 1000, max(1, n_valid), n_valid + 3}):
            if k > 16384:
                continue
            sw = sweep_for(w, k=k)
            sw.topk(0, n)
            torch.cuda.synchronize()
            gv, gi = sw.topk_host()
            parity.check_topk(gv, gi, oy, ov, 0, k)
            # tail entries past n_found are (+inf, 0xFFFFFFFF)
            nf = len(gi)
            if nf < k:
                assert torch.all(torch.isposinf(sw.values[nf:]))
                assert torch.all(sw.indices[nf:] == -1)
            say(f"  {w.name} k={k}: n_found {nf}")


def test_topk_every_list_length_of_the_merge_tree():
    """k from 1 to 4096 on the paper's convolution space (256 workgroup lists + the running
    result): list lengths 1 .. 32 (wave merge in LDS), 64 .. 512 (pair merge in registers),
    1024 and more (workgroup-wide merge)."""
    w = wl.paper_convolution()
    n = w.space.n_configs
    oy, ov, _ = oracle.predict_range(w.space, w.model, 0, n, threads=THREADS)
    for k in (1, 3, 17, 32, 33, 64, 65, 128, 129, 256, 257, 300, 512, 513, 1024, 4096):
        sw = sweep_for(w, k=k)
        sw.topk(0, n)
        torch.cuda.synchronize()
        gv, gi = sw.topk_host()
        assert len(gi) == k
        parity.check_topk(gv, gi, oy, ov, 0, k)
        # the same space in two disjoint calls, the second merging with the first's result
        cut = (n // 3) | 1
        sw.topk(cut, n - cut)
        sw.topk(0, cut, merge=True)
        torch.cuda.synchronize()
        gv2, gi2 = sw.topk_host()
        assert np.array_equal(gi, gi2) and np.array_equal(gv, gv2)


def test_topk_unconstrained_is_the_papers_unmasked_sweep():
    w = wl.conv_shaped()
    wu = wl.Workload("u", w.space.without_constraints(), w.model, w.k)
    n = wu.space.n_configs
    oy, ov, _ = oracle.predict_range(wu.space, wu.model, 0, n, threads=THREADS)
    assert ov.all()
    sw = sweep_for(wu)
    sw.topk(0, n)
    torch.cuda.synchronize()
    gv, gi = sw.topk_host()
    parity.check_topk(gv, gi, oy, ov, 0, wu.k)


def test_topk_chunked_merge_equals_one_call_any_order():
    w = wl.paper_raycasting()
    sp = w.space
    n = sp.n_configs
    sw = sweep_for(w)
    sw.topk(0, n)
    torch.cuda.synchronize()
    ref_v, ref_i = sw.topk_host()
    oy, ov, _ = oracle.predict_range(sp, w.model, 0, n, threads=THREADS)
    parity.check_topk(ref_v, ref_i, oy, ov, 0, w.k)
    bounds = [0, 1000, 1031, 200000, 200001, 500000, n]
    chunks = list(zip(bounds[:-1], bounds[1:]))
    for order in (list(range(len(chunks))), [5, 0, 3, 1, 4, 2]):
        sw2 = sweep_for(w)
        first = True
        for j in order:
            b, e = chunks[j]
            sw2.topk(b, e - b, merge=not first)
            first = False
        torch.cuda.synchronize()
        v, i = sw2.topk_host()
        # same kernels, same values: the merged result is bit-identical
        assert np.array_equal(i, ref_i) and np.array_equal(v, ref_v)
    # empty chunk keeps the running result; a fresh empty call gives an empty result
    sw2.topk(5, 0, merge=True)
    torch.cuda.synchronize()
    v, i = sw2.topk_host()
    assert np.array_equal(i, ref_i)
    sw2.topk(5, 0, merge=False)
    torch.cuda.synchronize()
    assert int(sw2.n_found.item()) == 0


def test_topk_repeatable_and_k_max():
    w = wl.conv_shaped()
    n = w.space.n_configs
    sw = sweep_for(w, k=16384)
    res = []
    for _ in range(3):
        sw.topk(0, n)
        torch.cuda.synchronize()
        res.append(sw.topk_host())
    for v, i in res[1:]:
        assert np.array_equal(i, res[0][1]) and np.array_equal(v, res[0][0])
    oy, ov, _ = oracle.predict_range(w.space, w.model, 0, n, threads=THREADS)
    parity.check_topk(res[0][0], res[0][1], oy, ov, 0, 16384)


@pytest.mark.parametrize("k", [1, 64, 300, 512, 1000])
def test_adversarial_order_descending_predictions(k):
    """Predictions that decrease with the index make every configuration pass
    the running threshold: exercises pool compaction under maximum pressure (k <= 512:
    selection in registers at every compaction; above: the workgroup-wide sort)."""
    sp = wl.Space("desc", [[float(v) for v in range(1, 65)]] * 3, [wl.SCALE_LINEAR] * 3)
    # y = -(256 sigmoid(2 x0) + sigmoid(2 x1)): non-increasing in the index, and every
    # new (x0, x1) group lies below everything seen before it
    m = wl.make_model([3, 8, 1], 1, 0)
    (Wh, bh), (wo, bo) = m.member_layers(0)
    Wh[:] = 0.0
    bh[:] = 0.0
    wo[:] = 0.0
    Wh[0, 0] = 2.0
    Wh[1, 1] = 2.0
    wo[0, 0] = -256.0
    wo[0, 1] = -1.0
    w = wl.Workload("desc", sp, m, k)
    n = sp.n_configs
    oy, ov, _ = oracle.predict_range(sp, m, 0, n, threads=THREADS)
    assert np.all(np.diff(oy.astype(np.float64)) <= 0)
    sw = sweep_for(w)
    sw.topk(0, n)
    torch.cuda.synchronize()
    gv, gi = sw.topk_host()
    parity.check_topk(gv, gi, oy, ov, 0, k)


@pytest.mark.parametrize("net", ["f32", "split16", "bf16"])
def test_topk_small_k_with_several_chunks_per_workgroup_on_wide_nets(net):
    """128-wide networks run in workgroups of 8 (fp32, two-plane f16) or 16 (bf16) waves;
    their candidate pools lie in the workspace (fp32; two-plane f16 from k = 512) or in LDS,
    and a sort of a workspace pool borrows the LDS that holds the weights.  2^19
    configurations are two to eight chunks for each of the 256 workgroups, so pools are cut
    back while the sweep goes on.  k on both sides of the limit of the selection in registers."""
    kw, tol = ({}, parity.TOL_FP32) if net == "f32" else _nets()[net]
    sp = wl.large().space
    m = wl.make_model([14, 128, 128, 1], 2, 77)
    begin, count = (5 << 21) + (3 << 18) + 12345, 1 << 19
    oy, ov, _ = oracle.predict_range(sp, m, begin, count, threads=THREADS)
    assert 0 < int(ov.sum()) < count
    for k in (1, 100, 512, 700):
        sw = sweep_for(wl.Workload("wide2", sp, m, k), **kw)
        sw.topk(begin, count)
        torch.cuda.synchronize()
        gv, gi = sw.topk_host()
        parity.check_topk(gv, gi, oy, ov, begin, k, tol=tol)
        say(f"  {net} k={k}: ok, {len(gi)} found")


def test_topk_and_predict_all_replay_from_a_hip_graph():
    """The library only enqueues kernels (no allocation, copy, memset or synchronisation),
    so a caller may capture its calls in a HIP graph.  A captured chunked top-k sweep and
    a captured predict_all are replayed several times with eager work and synchronisations
    between the replays; every replay must reproduce the eager result bit for bit."""
    w = wl.paper_raycasting()
    n = w.space.n_configs
    half = n // 2 + 12345                      # two ragged chunks merged on the device
    sw = sweep_for(w)
    sw.topk(0, half)
    sw.topk(half, n - half, merge=True)
    pred_eager, _ = sw.predict_all(0, n, want_mask=False)
    torch.cuda.synchronize()
    ref_v, ref_i = sw.topk_host()
    ref_pred = pred_eager.clone()
    oy, ov, _ = oracle.predict_range(w.space, w.model, 0, n, threads=THREADS)
    parity.check_topk(ref_v, ref_i, oy, ov, 0, w.k)

    pred = torch.empty(n, dtype=torch.float32, device=sw.device)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):              # warm-up on the capture stream
        sw.topk(0, half)
        sw.predict_all(0, n, want_mask=False, out=pred)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        sw.topk(0, half)
        sw.topk(half, n - half, merge=True)
        sw.predict_all(0, n, want_mask=False, out=pred)
    for rep in range(4):
        # eager work between replays: scribble over the outputs and run another sweep
        sw.values.fill_(-1.0)
        sw.indices.fill_(7)
        sw.n_found.fill_(0)
        pred.fill_(float("nan"))
        sw.topk(rep * 1000, 50000)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        gv, gi = sw.topk_host()
        assert np.array_equal(gv, ref_v) and np.array_equal(gi, ref_i), f"replay {rep}"
        assert torch.equal(pred, ref_pred), f"replay {rep}"


def test_profile_events_recorded_and_dropped():
    """Sweep timings are kept as pairs of events until they are read; switching profiling
    off drops the ones nobody read."""
    import paper_1506_00842_amd as T
    w = wl.conv_shaped()
    sw = sweep_for(w)
    T.tuner_profile_enable(True)
    try:
        T.tuner_profile_read()
        for _ in range(3):
            sw.topk(0, w.space.n_configs)
        sw.topk(5, 0)                                 # an empty range launches no sweep
        assert T.tuner_profile_pending() == 3
        ms, n = T.tuner_profile_read()
        assert n == 3 and 0.0 < ms < 1000.0 and T.tuner_profile_pending() == 0
        sw.topk(0, w.space.n_configs)
        assert T.tuner_profile_pending() == 1
    finally:
        T.tuner_profile_enable(False)
    assert T.tuner_profile_pending() == 0
    torch.cuda.synchronize()


# ------------------------------------------------------- prepared workspace ---
@pytest.mark.parametrize("maker,kw_name", [(wl.paper_raycasting, "f32"), (wl.conv_shaped, "f32"), (wl.large, "f32"),
                                           (wl.wide, "bf16"), (wl.paper_stereo, "split16"), (wl.tiny, "valu")])
def test_prepared_calls_equal_plain_calls(maker, kw_name):
    """tuner_prepare once, then prepared calls: the same bits as the plain entry points, call
    after call (the last workgroup of every sweep leaves the header ready for the next one),
    for short ranges, long ranges with the work queue and the live-chunk list, chunked running
    results, empty ranges, and predict_all in between."""
    import paper_1506_00842_amd as T
    kw = {"f32": {}, "bf16": dict(precision=T.TUNER_BF16_MFMA), "split16": dict(algo=T.TUNER_ALGO_SPLIT16),
          "valu": dict(algo=T.TUNER_ALGO_VALU)}[kw_name]
    w = maker()
    n = w.space.n_configs
    ref = sweep_for(w, **kw)
    sw = sweep_for(w, **kw)
    sw.prepare()
    long_count = min(n, (1 << 22) + 12345)
    calls = [(0, min(n, 100003), False), (n // 3, min(n - n // 3, 70001), True), (5, 0, True), (n - min(n, 4099), min(n, 4099), True),
             (0, long_count, False), (n - long_count, long_count, n > 2 * long_count), (7, 0, False), (0, min(n, 33), False)]
    for rep in range(2):
        for begin, count, merge in calls:
            ref.topk(begin, count, merge=merge)
            sw.topk(begin, count, merge=merge)
            torch.cuda.synchronize()
            assert torch.equal(sw.n_found, ref.n_found), (begin, count, merge)
            assert torch.equal(sw.values.view(torch.int32), ref.values.view(torch.int32)), (begin, count, merge)
            assert torch.equal(sw.indices, ref.indices), (begin, count, merge)
            if count and count <= 100003:
                p0, m0 = ref.predict_all(begin, count)
                p1, m1 = sw.predict_all(begin, count)
                torch.cuda.synchronize()
                assert torch.equal(p0.view(torch.int32), p1.view(torch.int32)) and torch.equal(m0, m1)
    p0, m0 = ref.predict_all(n - long_count, long_count)
    p1, m1 = sw.predict_all(n - long_count, long_count)
    torch.cuda.synchronize()
    assert torch.equal(p0.view(torch.int32), p1.view(torch.int32)) and torch.equal(m0, m1)
    # against the oracle too, on a range the oracle sweeps in a second
    begin, count = (n // 3, min(n - n // 3, 70001))
    sw.topk(begin, count)
    torch.cuda.synchronize()
    oy, ov, _ = oracle.predict_range(w.space, w.model, begin, count, threads=THREADS)
    gv, gi = sw.topk_host()
    parity.check_topk(gv, gi, oy, ov, begin, w.k, tol=TOL_BF16 if kw_name == "bf16" else parity.TOL_FP32)
    # the list evaluation repacks the weights: the wrapper falls back to plain calls after it
    idx = torch.arange(begin, begin + 1000, dtype=torch.int32, device=sw.device)
    sw.predict_indices(idx)
    assert not sw.prepared
    sw.topk(begin, count)
    torch.cuda.synchronize()
    gv2, gi2 = sw.topk_host()
    assert np.array_equal(gi, gi2) and np.array_equal(gv, gv2)


def test_prepared_and_static_calls_replay_from_a_hip_graph():
    """The callers the prepared and the static-scratch entry points are for: a captured
    sequence of sweeps replayed many times.  Every replay (with eager sweeps on the same
    workspace and scribbled outputs in between) reproduces the eager result bit for bit:
    the header's counters are back in their idle state after every call."""
    import paper_1506_00842_amd as T
    w = wl.paper_stereo()                      # long enough for the work queue and the live-chunk list
    n = w.space.n_configs
    cut = n // 2 + 4321
    sw = sweep_for(w)
    sw.topk(0, cut)
    sw.topk(cut, n - cut, merge=True)
    torch.cuda.synchronize()
    ref_v, ref_i = sw.values.clone(), sw.indices.clone()
    oy, ov, _ = oracle.predict_range(w.space, w.model, 0, n, threads=THREADS)
    gv, gi = sw.topk_host()
    parity.check_topk(gv, gi, oy, ov, 0, w.k)
    sw.prepare()
    sv = torch.empty_like(sw.values)
    si = torch.empty_like(sw.indices)
    sn = torch.zeros_like(sw.n_found)

    def static_calls():
        T.tuner_predict_topk_static(sw.space, sw.model, 0, cut, w.k, 0, sv, si, sn)
        T.tuner_predict_topk_static(sw.space, sw.model, cut, n - cut, w.k, 1, sv, si, sn)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):              # warm-up on the capture stream (first use of the static array too)
        sw.topk(0, cut)
        static_calls()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        sw.topk(0, cut)                        # prepared calls: sweep (+ classification) and one merge launch each
        sw.topk(cut, n - cut, merge=True)
        static_calls()
    for rep in range(4):
        sw.values.fill_(-1.0)
        sw.indices.fill_(7)
        sw.n_found.fill_(0)
        sv.fill_(-2.0)
        si.fill_(9)
        sw.topk(rep * 1000, 300000 + rep)      # eager prepared call on the same workspace
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(sw.values.view(torch.int32), ref_v.view(torch.int32)) and torch.equal(sw.indices, ref_i), f"replay {rep}"
        assert torch.equal(sv.view(torch.int32), ref_v.view(torch.int32)) and torch.equal(si, ref_i), f"replay {rep}"
        assert int(sn.item()) == w.k
