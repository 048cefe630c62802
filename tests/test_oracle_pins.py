"""Pins for the CPU oracle: values printed in the paper, closed forms,
invariants, reduction to numpy matrix algebra, and brute force on tiny spaces.
No GPU, no HIP library."""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- helpers ----
def enumerate_space(space):
    """Independent enumeration: itertools.product over the value lists gives the
    configurations in 'last parameter fastest' order."""
    digit_lists = [range(len(v)) for v in space.values]
    digs = np.array(list(itertools.product(*digit_lists)), dtype=np.int64)
    vals = np.array(list(itertools.product(*space.values)), dtype=np.float64)
    return digs.reshape(-1, space.n_params), vals.reshape(-1, space.n_params)


def numpy_features(space, vals):
    x = np.empty_like(vals)
    for p, lst in enumerate(space.values):
        t = np.log2(np.array(lst)) if space.scales[p] == wl.SCALE_LOG2 else np.array(lst, float)
        col = np.log2(vals[:, p]) if space.scales[p] == wl.SCALE_LOG2 else vals[:, p]
        lo, hi = t.min(), t.max()
        x[:, p] = (col - lo) / (hi - lo) if hi > lo else 0.0
    return x.astype(np.float32).astype(np.float64)


def numpy_valid(space, digs):
    ok = np.ones(len(digs), bool)
    off = space.offsets
    for c in range(space.n_constraints):
        s = np.zeros(len(digs), np.int64)
        for p in range(space.n_params):
            s += space.constraint_terms[c][off[p] + digs[:, p]]
        ok &= s <= space.constraint_bounds[c]
    return ok


def numpy_predict(space, model, x):
    total = np.zeros(len(x))
    for e in range(model.n_members):
        h = x
        layers = model.member_layers(e)
        for l, (W, b) in enumerate(layers):
            z = h @ W.astype(np.float64).T + b.astype(np.float64)
            h = 1.0 / (1.0 + np.exp(-z)) if l + 1 < len(layers) else z
        total += h[:, 0]
    return (total / model.n_members).astype(np.float32)


def full_sort_topk(yhat, valid, k):
    idx = np.nonzero(valid)[0]
    order = sorted(idx, key=lambda i: (float(yhat[i]), int(i)))[:k]
    return np.array([yhat[i] for i in order], np.float32), np.array(order, np.uint64)


# ------------------------------------------------------------------- P1 ------
def test_paper_space_sizes():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "paper_space_sizes.txt"))
            if l.strip() and not l.startswith("#")]
    makers = {"convolution": wl.paper_convolution, "raycasting": wl.paper_raycasting,
              "stereo": wl.paper_stereo}
    for name, kilo, evaluated, pct, *rad in rows:
        sp = makers[name]().space
        assert list(sp.radices) == [int(r) for r in rad]
        n = sp.n_configs
        assert n // 1000 == int(kilo)                       # "131K, 655K and 2359K"
        assert round(100.0 * int(evaluated) / n, 1) == float(pct)
        # last index decodes to the last value of every list (non-power-of-two radices too)
        assert list(oracle.digits(sp, n - 1)) == [r - 1 for r in sp.radices]
    assert wl.paper_convolution().space.n_configs == 131072
    assert wl.paper_raycasting().space.n_configs == 655360
    assert wl.paper_stereo().space.n_configs == 2359296


def test_benchmark_space_sizes():
    assert wl.tiny().space.n_configs == 256
    assert wl.conv_shaped().space.n_configs == 393216
    assert wl.large().space.n_configs == 1 << 27
    assert wl.large_as_written().space.n_configs == 1 << 26
    assert wl.streamed().space.n_configs == 1 << 32


# ------------------------------------------------------------------- P2/P3 ---
@pytest.mark.parametrize("maker", [wl.tiny, lambda: wl.random_small(3), lambda: wl.random_small(8)])
def test_decode_encode_roundtrip_small(maker):
    sp = maker().space
    digs, _ = enumerate_space(sp)
    for i in range(sp.n_configs):
        d = oracle.digits(sp, i)
        assert list(d) == list(digs[i])
        assert oracle.index(sp, d) == i


@pytest.mark.parametrize("maker", [wl.conv_shaped, wl.large, wl.streamed, wl.paper_stereo])
def test_decode_encode_roundtrip_random(maker):
    sp = maker().space
    st = wl.Stream(123)
    n = sp.n_configs
    for i in [0, 1, n - 1, n // 2, n // 3] + [int(v) for v in st.integers(2000, n)]:
        d = oracle.digits(sp, i)
        assert all(0 <= d[p] < sp.radices[p] for p in range(sp.n_params))
        assert oracle.index(sp, d) == i
    # encode then decode
    for _ in range(200):
        d = [int(st.integers(1, int(r))[0]) for r in sp.radices]
        assert list(oracle.digits(sp, oracle.index(sp, d))) == d


@pytest.mark.parametrize("maker", [wl.conv_shaped, wl.paper_raycasting, wl.streamed])
def test_decode_closed_forms(maker):
    sp = maker().space
    rad = [int(r) for r in sp.radices]
    P = len(rad)
    assert list(oracle.digits(sp, 0)) == [0] * P
    one = oracle.digits(sp, 1)
    assert list(one) == [0] * (P - 1) + [1]
    assert list(oracle.digits(sp, sp.n_configs - 1)) == [r - 1 for r in rad]
    stride = 1
    for p in range(P - 1, -1, -1):
        if rad[p] > 1:
            expect = [0] * P
            expect[p] = 1
            assert list(oracle.digits(sp, stride)) == expect
        stride *= rad[p]


# ------------------------------------------------------------------- P4 ------
def test_feature_closed_forms():
    sp = wl.tiny().space
    lut = oracle.feature_lut(sp)
    third = np.float32(1.0 / 3.0)
    two_thirds = np.float32(2.0 / 3.0)
    assert list(lut[0:4]) == [0.0, third, two_thirds, 1.0]      # {1,2,4,8} log2
    assert list(lut[4:8]) == [0.0, third, two_thirds, 1.0]
    assert list(lut[8:10]) == [0.0, 1.0]                         # {0,1} linear
    assert list(lut[10:18]) == [np.float32((v - 1) / 7.0) for v in range(1, 9)]
    for maker in (wl.conv_shaped, wl.large, wl.streamed, wl.paper_stereo):
        s = maker().space
        l = oracle.feature_lut(s)
        for p, o in enumerate(s.offsets):
            assert l[o] == 0.0 and l[o + s.radices[p] - 1] == 1.0
            assert np.all(np.diff(l[o:o + s.radices[p]]) > 0)
    # a one-value list and a constant list map to 0
    deg = wl.Space("deg", [[5.0], [2.0, 2.0]], [wl.SCALE_LOG2, wl.SCALE_LINEAR])
    assert list(oracle.feature_lut(deg)) == [0.0, 0.0, 0.0]


def test_streamed_rule_is_a_product_bound():
    """The fixed-point log2 terms of the 2**32 space encode v0*v1*v2 <= 1024."""
    sp = wl.streamed().space
    t = sp.constraint_terms[0][:16]
    for a in range(16):
        for b in range(16):
            for c in range(16):
                assert (int(t[a]) + int(t[b]) + int(t[c]) <= (10 << 20)) == ((a + 1) * (b + 1) * (c + 1) <= 1024)


# ------------------------------------------------------------------- P5 ------
def test_mask_count_conv_exact():
    w = wl.conv_shaped()
    _, valid, _ = oracle.predict_range(w.space, None, 0, w.space.n_configs, want_yhat=False)
    assert int(valid.sum()) == 331_776 == w.n_valid
    assert 331_776 == 54 * 6144          # 54 of 64 (wg_x, wg_y) pairs, times the rest
    _, v2, _ = oracle.predict_range(w.space.without_constraints(), None, 0, 4096, want_yhat=False)
    assert int(v2.sum()) == 4096


def test_mask_count_paper_spaces():
    """Work-group rule wg_x * wg_y <= 1024 keeps 54 of the 64 (wg_x, wg_y) pairs."""
    for maker in (wl.paper_convolution, wl.paper_raycasting, wl.paper_stereo):
        w = maker()
        n = w.space.n_configs
        _, valid, _ = oracle.predict_range(w.space, None, 0, n, threads=8, want_yhat=False)
        assert int(valid.sum()) == w.n_valid == n * 54 // 64


def test_mask_count_large_analytic():
    """Digits 0..3 decide validity and are constant over aligned blocks of
    2**15 indices: count valid blocks at their first index."""
    w = wl.large()
    sp = w.space
    block = 1 << 15
    n_valid = 0
    for b in range(sp.n_configs // block):
        _, v, _ = oracle.predict_range(sp, None, b * block, 1, want_yhat=False)
        n_valid += int(v[0]) * block
    assert n_valid == 63_700_992 == 54 * 36 * (1 << 15) == w.n_valid
    # inside a block the mask really is constant (spot check)
    for b in (0, 7, 4095):
        _, v, _ = oracle.predict_range(sp, None, b * block, block, want_yhat=False)
        assert v.min() == v.max()


def test_mask_count_streamed_analytic():
    """Rules touch parameters 0..9 only; the 22 low bits (parameters 10..19 and
    below) are free.  Count over the 2**20 high-digit combinations by stepping
    one index per combination."""
    w = wl.streamed()
    sp = w.space
    low = 1 << 10                                   # parameters 10..19: 10 flags
    # product structure: rule 0 on (p0,p1,p2), rule 1 on (p3,p4,p5), rule 2 on (p6..p9)
    digs, _ = enumerate_space(wl.Space("s", sp.values[:3], sp.scales[:3]))
    t = sp.constraint_terms[0][:16].astype(np.int64)
    c0 = int(np.sum(t[digs[:, 0]] + t[digs[:, 1]] + t[digs[:, 2]] <= (10 << 20)))
    c1 = sum(1 for a in range(4) for b in range(4) for c in range(4) if a + b + c <= 7)
    c2 = sum(1 for f in itertools.product((0, 1), repeat=4) if sum(f) <= 3)
    assert (c0, c1, c2) == (3268, 60, 15)
    assert c0 * c1 * c2 * low == 3_011_788_800 == w.n_valid
    # the oracle's mask agrees with the product form on random indices
    st = wl.Stream(5)
    for i in [int(v) for v in st.integers(3000, sp.n_configs)]:
        _, v, d = oracle.predict_range(sp, None, i, 1, want_yhat=False, want_digits=True)
        d = d[0]
        ok = (t[d[0]] + t[d[1]] + t[d[2]] <= (10 << 20)) and (d[3] + d[4] + d[5] <= 7) \
            and (d[6] + d[7] + d[8] + d[9] <= 3)
        assert bool(v[0]) == bool(ok)


# ------------------------------------------------------------------- P6-P8 ---
def test_zero_weights_give_mean_output_bias():
    w = wl.conv_shaped()
    m = w.model
    z = wl.Model(m.widths, m.n_members, np.zeros_like(m.weights))
    fpm = z.floats_per_member
    biases = np.array([0.25, -1.5, 3.0, 0.125, 7.0, -2.0, 0.5, 1.0], np.float32)
    for e in range(z.n_members):
        z.weights[(e + 1) * fpm - 1] = biases[e]
    yhat, valid, _ = oracle.predict_range(w.space, z, 1000, 5000)
    expect = np.float32(np.float64(biases.astype(np.float64).sum()) / 8.0)
    assert np.all(yhat[valid == 1] == expect)
    assert np.all(np.isposinf(yhat[valid == 0]))


def test_single_unit_closed_form():
    gold = {}
    for line in open(os.path.join(GOLDEN, "closed_forms.txt")):
        if line.startswith("sigmoid"):
            _, t, v = line.split()
            gold[float(t)] = float(v)
    sp = wl.Space("one", [[0.0, 1.0, 2.0]], [wl.SCALE_LINEAR])     # features 0, 0.5, 1
    # y = w_o * sigmoid(w1 x + b1) + b_o
    for (w1, b1, wo, bo) in [(2.0, -1.0, 1.0, 0.0), (2.0, 0.0, 3.0, -1.0), (-2.0, 1.0, 0.5, 0.25)]:
        m = wl.Model([1, 1, 1], 1, np.array([w1, b1, wo, bo], np.float32))
        yhat, _, _ = oracle.predict_range(sp, m, 0, 3)
        for j, x in enumerate((0.0, 0.5, 1.0)):
            t = w1 * x + b1
            assert t in gold
            assert yhat[j] == np.float32(wo * gold[t] + bo)
    # sigma(0) = 1/2 exactly
    m = wl.Model([1, 1, 1], 1, np.array([1.0, 0.0, 1.0, 0.0], np.float32))
    assert oracle.predict_range(sp, m, 0, 1)[0][0] == 0.5


def test_constant_net_and_saturation():
    w = wl.tiny()
    m = wl.Model(w.model.widths, 1, w.model.weights.copy())
    W1 = m.member_layers(0)[0][0]
    W1[:] = 0.0
    yhat, _, _ = oracle.predict_range(w.space, m, 0, 256)
    assert np.all(yhat == yhat[0])
    for big, sig in ((1e4, 1.0), (-1e4, 0.0)):
        m2 = wl.Model([4, 16, 1], 1, np.zeros_like(m.weights))
        (W1, b1), (wo, bo) = m2.member_layers(0)
        b1[:] = big
        wo[:] = 1.0
        yhat, _, _ = oracle.predict_range(w.space, m2, 0, 256)
        assert np.all(np.isfinite(yhat)) and np.all(yhat == np.float32(16 * sig))


# ------------------------------------------------------------------- P9 ------
def test_ensemble_mean_invariants():
    w = wl.conv_shaped()
    m = w.model
    fpm = m.floats_per_member
    one = wl.Model(m.widths, 1, m.weights[:fpm].copy())
    rep = wl.Model(m.widths, 4, np.tile(m.weights[:fpm], 4))
    y1, v, _ = oracle.predict_range(w.space, one, 5000, 3000)
    y4, _, _ = oracle.predict_range(w.space, rep, 5000, 3000)
    assert np.array_equal(y1, y4)
    perm = np.concatenate([m.weights[e * fpm:(e + 1) * fpm] for e in (3, 0, 7, 1, 6, 2, 5, 4)])
    ya, _, _ = oracle.predict_range(w.space, m, 5000, 3000)
    yb, _, _ = oracle.predict_range(w.space, wl.Model(m.widths, 8, perm), 5000, 3000)
    ok = v == 1
    ulp = np.spacing(np.abs(ya[ok]))
    assert np.all(np.abs(ya[ok] - yb[ok]) <= ulp)


# ------------------------------------------------------------------- P10 -----
def _check_against_numpy(w, atol=0.0):
    sp, m = w.space, w.model
    digs, vals = enumerate_space(sp)
    yhat, valid, d = oracle.predict_range(sp, m, 0, sp.n_configs, threads=4, want_digits=True)
    assert np.array_equal(d, digs)
    ok = numpy_valid(sp, digs)
    assert np.array_equal(valid.astype(bool), ok)
    ref = numpy_predict(sp, m, numpy_features(sp, vals))
    assert np.all(np.isposinf(yhat[~ok]))
    # BLAS sums in a different order than the plain loop: allow 1 fp32 ulp
    assert np.all(np.abs(yhat[ok] - ref[ok]) <= np.spacing(np.abs(ref[ok])))


@pytest.mark.parametrize("seed", [1, 2, 3, 4, 5])
def test_matrix_algebra_small(seed):
    _check_against_numpy(wl.random_small(seed, n_hidden_layers=1 + seed % 2))


def test_matrix_algebra_tiny_and_conv():
    _check_against_numpy(wl.tiny())
    _check_against_numpy(wl.conv_shaped())


def test_matrix_algebra_two_hidden_slice():
    """Slice of the 2**27 space with the 14-64-64-1 ensemble, features from an
    independent digit computation."""
    w = wl.large()
    sp, m = w.space, w.model
    begin, count = (37 << 15) + 12345, 4096
    yhat, valid, d = oracle.predict_range(sp, m, begin, count, want_digits=True)
    idx = np.arange(begin, begin + count, dtype=np.int64)
    digs = np.zeros((count, sp.n_params), np.int64)
    stride = 1
    for p in range(sp.n_params - 1, -1, -1):
        digs[:, p] = (idx // stride) % sp.radices[p]
        stride *= int(sp.radices[p])
    assert np.array_equal(d, digs)
    vals = np.stack([np.array(sp.values[p])[digs[:, p]] for p in range(sp.n_params)], axis=1)
    ok = numpy_valid(sp, digs)
    assert np.array_equal(valid.astype(bool), ok) and ok.any()
    ref = numpy_predict(sp, m, numpy_features(sp, vals))
    assert np.all(np.abs(yhat[ok] - ref[ok]) <= np.spacing(np.abs(ref[ok])))


def test_threaded_driver_equals_single_thread():
    w = wl.conv_shaped()
    a = oracle.predict_range(w.space, w.model, 777, 20001, threads=1, want_digits=True)
    b = oracle.predict_range(w.space, w.model, 777, 20001, threads=5, want_digits=True)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


# ------------------------------------------------- evaluation at a list -------
def _digits_by_divmod(sp, idx):
    digs = np.zeros((len(idx), sp.n_params), np.int64)
    q = np.asarray(idx, dtype=np.uint64).astype(object)        # Python integers: no 64-bit surprises
    for p in range(sp.n_params - 1, -1, -1):
        r = int(sp.radices[p])
        digs[:, p] = [int(v) % r for v in q]
        q = np.array([int(v) // r for v in q], dtype=object)
    return digs


@pytest.mark.parametrize("maker,n_list", [(wl.conv_shaped, 3000), (wl.large, 2000), (wl.streamed, 1500),
                                          (wl.paper_raycasting, 2500)])
def test_predict_indices_against_numpy_algebra_at_scattered_indices(maker, n_list):
    """The list evaluation (used to judge every index a top-k sweep returns) against numpy
    matrix algebra with digits from plain divmod, at indices scattered over the whole space,
    unsorted, with repeats, for one and several threads."""
    w = maker()
    sp, m = w.space, w.model
    n = sp.n_configs
    st = wl.Stream(99)
    idx = st.integers(n_list, n).astype(np.uint64)
    idx[::7] = idx[3]                                          # repeats
    idx[:4] = [0, n - 1, 1, n - 2]                             # the ends of the space
    digs = _digits_by_divmod(sp, idx)
    vals = np.stack([np.array(sp.values[p])[digs[:, p]] for p in range(sp.n_params)], axis=1)
    ok = numpy_valid(sp, digs)
    assert ok.any() and (~ok).any()                            # valid and invalid entries in the list
    ref = numpy_predict(sp, m, numpy_features(sp, vals))
    for threads in (1, 3, 16):
        y, v = oracle.predict_indices(sp, m, idx, threads=threads)
        assert np.array_equal(v.astype(bool), ok)
        assert np.all(np.isposinf(y[~ok]))
        assert np.all(np.abs(y[ok] - ref[ok]) <= np.spacing(np.abs(ref[ok])))
        if threads == 1:
            y1 = y
        assert np.array_equal(y, y1)                           # the thread split changes nothing


def test_predict_indices_equals_predict_range():
    w = wl.conv_shaped()
    sp, m = w.space, w.model
    begin, count = 5 * 49152 + 6 * 6144 - 10000, 20011       # wg_x = 32, wg_y from 32 into 64: valid, then not
    ry, rv, _ = oracle.predict_range(sp, m, begin, count)
    ar = np.arange(begin, begin + count, dtype=np.uint64)
    for threads in (1, 4):
        y, v = oracle.predict_indices(sp, m, ar, threads=threads)                 # the range as a list
        assert np.array_equal(y, ry) and np.array_equal(v, rv)
    perm = np.argsort(wl.Stream(5).uniform(count))                                # shuffled
    y, v = oracle.predict_indices(sp, m, ar[perm], threads=3)
    assert np.array_equal(y, ry[perm]) and np.array_equal(v, rv[perm])
    rep = np.concatenate([ar[:100], ar[:100], ar[50:60]])                         # repeats
    y, v = oracle.predict_indices(sp, m, rep, threads=2)
    assert np.array_equal(y, np.concatenate([ry[:100], ry[:100], ry[50:60]]))
    inv = ar[rv == 0][:50]                                                        # invalid ones only
    assert len(inv) == 50
    y, v = oracle.predict_indices(sp, m, inv, threads=2)
    assert np.all(np.isposinf(y)) and not v.any()
    y, v = oracle.predict_indices(sp, m, np.zeros(0, np.uint64), threads=4)       # empty list
    assert len(y) == 0 and len(v) == 0
    y, v = oracle.predict_indices(sp, m, ar[:3], threads=16)                      # more threads than entries
    assert np.array_equal(y, ry[:3])


# ------------------------------------------------------------------- P11 -----
@pytest.mark.parametrize("seed", [1, 2, 3, 4, 5, 6])
def test_topk_brute_force(seed):
    w = wl.random_small(seed)
    sp = w.space
    yhat, valid, _ = oracle.predict_range(sp, w.model, 0, sp.n_configs)
    nv = int(valid.sum())
    for k in (1, 2, w.k, nv, nv + 5):
        vals, idx = oracle.select_topk(yhat, valid, 0, k)
        rv, ri = full_sort_topk(yhat, valid, k)
        assert np.array_equal(vals, rv) and np.array_equal(idx, ri)
        assert len(idx) == min(k, nv)
    if nv:
        vals, idx = oracle.select_topk(yhat, valid, 0, 1)
        vi = np.nonzero(valid)[0]
        assert idx[0] == vi[np.argmin(yhat[vi])]


def test_topk_ties_break_by_index():
    yhat = np.array([2.0, 1.0, 1.0, 3.0, 1.0, 0.5, 1.0], np.float32)
    valid = np.array([1, 1, 1, 1, 0, 1, 1], np.uint8)
    vals, idx = oracle.select_topk(yhat, valid, 100, 3)
    assert list(idx) == [105, 101, 102] and list(vals) == [0.5, 1.0, 1.0]
    # all equal: the first k indices
    vals, idx = oracle.select_topk(np.ones(50, np.float32), None, 0, 7)
    assert list(idx) == list(range(7))
    assert len(oracle.select_topk(yhat, valid, 0, 0)[0]) == 0


def test_topk_tiny_config():
    w = wl.tiny()
    vals, idx = oracle.topk(w.space, w.model, 0, 256, w.k)
    yhat, valid, _ = oracle.predict_range(w.space, w.model, 0, 256)
    rv, ri = full_sort_topk(yhat, valid, w.k)
    assert np.array_equal(idx, ri) and np.array_equal(vals, rv)


# ------------------------------------------------------------------- P12 -----
def test_topk_monotone_map_and_chunking():
    w = wl.conv_shaped()
    sp, m = w.space, w.model
    n = sp.n_configs
    yhat, valid, _ = oracle.predict_range(sp, m, 0, n, threads=8)
    vals, idx = oracle.select_topk(yhat, valid, 0, w.k)
    # positive affine map of every member's output layer: a*w_o, a*b_o + c
    a, c = 2.0, 3.0            # exact in binary: ordering preserved up to final rounding ties
    m2 = wl.Model(m.widths, m.n_members, m.weights.copy())
    for e in range(m2.n_members):
        wo, bo = m2.member_layers(e)[-1]
        wo *= np.float32(a)
        bo[:] = bo * np.float32(a) + np.float32(c)
    y2, _, _ = oracle.predict_range(sp, m2, 0, n, threads=8)
    v2, i2 = oracle.select_topk(y2, valid, 0, w.k)
    # compare as sets away from the boundary (rounding may create/break ties at the k-th value)
    assert set(idx[:-5]) <= set(i2) and set(i2[:-5]) <= set(idx)
    # chunked selection with merging == unchunked, any chunk order
    chunks = [(0, 100000), (100000, 150000), (250000, n - 250000)]
    for order in ([0, 1, 2], [2, 0, 1]):
        cand_v, cand_i = [], []
        for j in order:
            b, cnt = chunks[j]
            cv, ci = oracle.select_topk(yhat[b:b + cnt], valid[b:b + cnt], b, w.k)
            cand_v.append(cv); cand_i.append(ci)
        cv = np.concatenate(cand_v); ci = np.concatenate(cand_i)
        order2 = sorted(range(len(cv)), key=lambda t: (float(cv[t]), int(ci[t])))[:w.k]
        assert np.array_equal(ci[order2], idx) and np.array_equal(cv[order2], vals)


def test_generator_is_reproducible():
    a = wl.make_model([4, 16, 1], 1, 0).weights
    b = wl.make_model([4, 16, 1], 1, 0).weights
    assert np.array_equal(a, b) and a.dtype == np.float32 and len(a) == 97
    c = wl.make_model([4, 16, 1], 1, 1).weights
    assert not np.array_equal(a, c)
    big = wl.make_model([14, 64, 64, 1], 4, 2)
    assert len(big.weights) == 20740 and big.macs_per_config == 20224 and big.sigmoids_per_config == 512
    W1 = big.member_layers(0)[0][0]
    assert abs(float(W1.std()) - 1 / math.sqrt(14)) < 0.02
    assert wl.wide().model.macs_per_config == 292864
    assert wl.streamed().model.macs_per_config == 43520


# ------------------------------------------------------------ sanitizers -----
def test_oracle_runs_clean_under_address_and_undefined_behaviour_sanitizers():
    """Every oracle entry point on the 256-configuration space in a build with
    -fsanitize=address,undefined and no Python in the process (oracle/sanitize_driver.cpp)."""
    import subprocess
    from oracle.build import build_sanitized
    exe = build_sanitized()
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "oracle sanitizer run ok" in r.stdout
    assert "ERROR" not in r.stderr and "runtime error" not in r.stderr
