"""Pins for the CPU oracle's sampler, ensemble training, accuracy metric and
second-stage pick: brute force from the definitions, closed forms, finite
differences and reverse-mode automatic differentiation of an independently
written loss, and invariants.  No GPU, no HIP library."""
import math
import os

import numpy as np
import pytest

import oracle
import workloads as wl
from workloads.synthetic_benchmark import SyntheticBenchmark, initial_weights, parts_round_robin

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
M64 = (1 << 64) - 1


# ---------------------------------------------------------------- helpers ----
def py_splitmix64(seed: int, counter: int) -> int:
    z = (seed + (counter + 1) * 0x9E3779B97F4A7C15) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def np_digits(space, indices):
    return np.stack(np.unravel_index(np.asarray(indices, dtype=np.int64),
                                     tuple(int(r) for r in space.radices)), axis=1)


def np_valid(space, digs):
    ok = np.ones(len(digs), bool)
    off = space.offsets
    for c in range(space.n_constraints):
        s = np.zeros(len(digs), np.int64)
        for p in range(space.n_params):
            s += space.constraint_terms[c][off[p] + digs[:, p]]
        ok &= s <= space.constraint_bounds[c]
    return ok


def np_features(space, digs):
    x = np.empty(digs.shape, np.float64)
    for p, lst in enumerate(space.values):
        t = np.log2(np.array(lst)) if space.scales[p] == wl.SCALE_LOG2 else np.array(lst, float)
        lo, hi = t.min(), t.max()
        col = (t - lo) / (hi - lo) if hi > lo else np.zeros_like(t)
        x[:, p] = col.astype(np.float32).astype(np.float64)[digs[:, p]]
    return x


def usable_mask(space, indices, times):
    t = np.asarray(times, np.float32)
    return np_valid(space, np_digits(space, indices)) & np.isfinite(t) & (t > 0)


def split(w, P, H):
    W1 = w[:H * P].reshape(H, P)
    b1 = w[H * P:H * P + H]
    wo = w[H * P + H:H * P + 2 * H]
    bo = w[H * P + 2 * H]
    return W1, b1, wo, bo


def np_loss(w, x, target, P, H):
    """Mean squared error of one network, written from the definition (float64)."""
    W1, b1, wo, bo = split(np.asarray(w, np.float64), P, H)
    h = 1.0 / (1.0 + np.exp(-(x @ W1.T + b1)))
    y = h @ wo + bo
    return float(np.mean((y - target) ** 2))


def small_problem(seed=3, n=60, E=3, H=4):
    w = wl.random_small(seed, max_configs=600, n_constraints=1)
    sp = w.space
    idx = oracle.sample_valid(sp, seed, n, 40 * n)
    assert len(idx) >= 20
    bm = SyntheticBenchmark(sp, seed, fail_fraction=0.1)
    t = bm.times(idx)
    parts = parts_round_robin(len(idx), E)
    w0 = initial_weights(E, sp.n_params, H, seed + 100)
    return sp, idx, t, parts, w0, E, H


# ---------------------------------------------------------------- sampler ----
def test_splitmix64_published_vector():
    """First outputs of splitmix64 from state 1234567 as published with the
    reference implementation (Steele, Lea & Flood 2014; Vigna's splitmix64.c test
    values): output n of the sequential generator = mix(seed + n * gamma)."""
    with open(os.path.join(GOLDEN, "splitmix64_vector.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    seed = int(rows[0][1])
    expected = [int(r[0]) for r in rows[1:]]
    assert [py_splitmix64(seed, c) for c in range(len(expected))] == expected


@pytest.mark.parametrize("maker,seed,n,max_draws", [
    (wl.tiny, 1, 40, 200), (wl.conv_shaped, 2, 500, 900), (wl.paper_stereo, 3, 300, 400),
    (lambda: wl.random_small(5, n_constraints=2), 4, 50, 5000),
    (lambda: wl.random_small(9, n_constraints=2), 5, 10_000, 3000),   # space smaller than n
])
def test_sampler_is_the_definition(maker, seed, n, max_draws):
    sp = maker().space
    N = sp.n_configs
    draws = [(py_splitmix64(seed, c) * N) >> 64 for c in range(max_draws)]
    ok = np_valid(sp, np_digits(sp, draws))
    seen, expect = set(), []
    for d, v in zip(draws, ok):
        if len(expect) == n:
            break
        if v and d not in seen:
            seen.add(d)
            expect.append(d)
    got = oracle.sample_valid(sp, seed, n, max_draws)
    assert got.tolist() == expect
    assert len(set(got.tolist())) == len(got)
    # a shorter sample is a prefix of a longer one
    if len(got) > 3:
        assert oracle.sample_valid(sp, seed, len(got) // 2, max_draws).tolist() == expect[:len(got) // 2]


def test_sampler_64_bit_seed_and_large_space():
    sp = wl.streamed().space           # 2^32 configurations: index = top 32 bits of the draw
    seed = 0xFEDCBA9876543210
    got = oracle.sample_valid(sp, seed, 64, 4096)
    draws = [py_splitmix64(seed, c) >> 32 for c in range(4096)]
    ok = np_valid(sp, np_digits(sp, draws))
    expect = []
    for d, v in zip(draws, ok):
        if v and d not in expect:
            expect.append(d)
    assert got.tolist() == expect[:64]


# --------------------------------------------------------------- training ----
def test_first_step_from_zero_weights_closed_form():
    """All weights zero: every output is 0 and every hidden unit 0.5, so
    L = mean(ln t)^2... precisely mean((ln t)^2); dL/db_o = -2 mean(ln t),
    dL/dw_o[j] = -mean(ln t), all other gradients vanish (they carry a factor w_o = 0).
    One step of size eta gives b_o = 2 eta m, w_o = eta m, m = mean of ln t over the
    network's own training samples."""
    sp, idx, t, parts, _w0, E, H = small_problem()
    P = sp.n_params
    per = H * P + 2 * H + 1
    eta = 0.25
    w1, loss = oracle.train_ensemble(sp, E, H, idx, t, parts, np.zeros(E * per, np.float32), 1, eta, 0.7)
    use = usable_mask(sp, idx, t)
    for e in range(E):
        lt = np.log(t[use & (parts != e)].astype(np.float64))
        m = lt.mean()
        W1, b1, wo, bo = split(w1[e * per:(e + 1) * per], P, H)
        assert np.all(W1 == 0) and np.all(b1 == 0)
        np.testing.assert_allclose(wo, np.full(H, eta * m), rtol=1e-6)
        np.testing.assert_allclose(bo, 2 * eta * m, rtol=1e-6)
        np.testing.assert_allclose(loss[e, 0], np.mean(lt ** 2), rtol=1e-12)


def test_gradient_matches_finite_differences_of_the_definition():
    sp, idx, t, parts, w0, E, H = small_problem(seed=4)
    P = sp.n_params
    per = H * P + 2 * H + 1
    eta = 1.0
    w1, loss = oracle.train_ensemble(sp, E, H, idx, t, parts, w0, 1, eta, 0.0)
    use = usable_mask(sp, idx, t)
    x_all = np_features(sp, np_digits(sp, idx))
    for e in range(E):
        sel = use & (parts != e)
        x, target = x_all[sel], np.log(t[sel].astype(np.float64))
        we = w0[e * per:(e + 1) * per].astype(np.float64)
        np.testing.assert_allclose(loss[e, 0], np_loss(we, x, target, P, H), rtol=1e-12)
        grad = (we - w1[e * per:(e + 1) * per].astype(np.float64)) / eta
        fd = np.empty(per)
        for q in range(per):
            hq = 1e-5
            wp, wm = we.copy(), we.copy()
            wp[q] += hq
            wm[q] -= hq
            fd[q] = (np_loss(wp, x, target, P, H) - np_loss(wm, x, target, P, H)) / (2 * hq)
        scale = np.abs(fd).max()
        assert scale > 1e-3
        # the step is read back from fp32 weights: resolution 6e-8 * |w| / eta
        assert np.abs(grad - fd).max() <= 2e-6 * max(scale, 1.0)


def test_trajectory_matches_reverse_mode_autodiff():
    """The same definition in plain PyTorch CPU float64 with autograd, stepped with
    v <- mu v - eta g, w <- w + v: weights after 40 epochs and the whole loss history."""
    torch = pytest.importorskip("torch")
    sp, idx, t, parts, w0, E, H = small_problem(seed=6, n=80, E=2, H=5)
    P = sp.n_params
    per = H * P + 2 * H + 1
    epochs, eta, mu = 40, 0.0625, 0.875      # exactly representable in fp32 (the oracle takes fp32 options)
    w_or, loss_or = oracle.train_ensemble(sp, E, H, idx, t, parts, w0, epochs, eta, mu)
    use = usable_mask(sp, idx, t)
    x_all = np_features(sp, np_digits(sp, idx))
    for e in range(E):
        sel = use & (parts != e)
        x = torch.tensor(x_all[sel], dtype=torch.float64)
        target = torch.tensor(np.log(t[sel].astype(np.float64)))
        w = torch.tensor(w0[e * per:(e + 1) * per].astype(np.float64), requires_grad=True)
        v = torch.zeros(per, dtype=torch.float64)
        hist = []
        for ep in range(epochs + 1):
            W1 = w[:H * P].reshape(H, P)
            h = torch.sigmoid(x @ W1.T + w[H * P:H * P + H])
            y = h @ w[H * P + H:H * P + 2 * H] + w[H * P + 2 * H]
            loss = torch.mean((y - target) ** 2)
            hist.append(float(loss.detach()))
            if ep == epochs:
                break
            (g,) = torch.autograd.grad(loss, w)
            with torch.no_grad():
                v = mu * v - eta * g
                w += v
        np.testing.assert_allclose(loss_or[e], np.array(hist), rtol=1e-9)
        np.testing.assert_allclose(w_or[e * per:(e + 1) * per], w.detach().numpy().astype(np.float32),
                                   rtol=2e-6, atol=1e-7)
        assert hist[-1] < 0.5 * hist[0]          # it does learn


def test_each_network_ignores_its_own_part_and_unusable_samples():
    sp, idx, t, parts, w0, E, H = small_problem(seed=8, n=90)
    t = t.copy()
    t[::7] = -1.0                      # some failed runs for certain
    P = sp.n_params
    per = H * P + 2 * H + 1
    ref, loss_ref = oracle.train_ensemble(sp, E, H, idx, t, parts, w0, 15, 0.1, 0.5)
    # (1) changing the times of part e leaves network e unchanged, bit for bit
    for e in range(E):
        t2 = t.copy()
        t2[parts == e] *= 3.0
        got, _ = oracle.train_ensemble(sp, E, H, idx, t2, parts, w0, 15, 0.1, 0.5)
        assert np.array_equal(got[e * per:(e + 1) * per], ref[e * per:(e + 1) * per])
        others = [q for q in range(E) if q != e]
        assert any(not np.array_equal(got[q * per:(q + 1) * per], ref[q * per:(q + 1) * per]) for q in others)
    # (2) failed runs (-1, 0, NaN, inf) and statically invalid configurations do not count:
    #     dropping them from the arrays gives the same weights and losses
    use = usable_mask(sp, idx, t)
    assert (~use).any()
    t3 = t.copy()
    bad = np.nonzero(~use)[0]
    for n_, b in enumerate(bad):
        t3[b] = [-1.0, 0.0, np.nan, np.inf][n_ % 4]
    got3, loss3 = oracle.train_ensemble(sp, E, H, idx, t3, parts, w0, 15, 0.1, 0.5)
    got4, loss4 = oracle.train_ensemble(sp, E, H, idx[use], t[use], parts[use], w0, 15, 0.1, 0.5)
    assert np.array_equal(got3, ref) and np.array_equal(got4, ref)
    assert np.array_equal(loss3, loss_ref) and np.array_equal(loss4, loss_ref)
    # an invalid configuration with a good time is ignored as well
    all_idx = np.arange(sp.n_configs)
    invalid = all_idx[~np_valid(sp, np_digits(sp, all_idx))]
    if len(invalid):
        idx5 = np.concatenate([idx, invalid[:5].astype(np.uint64)])
        t5 = np.concatenate([t, np.full(len(invalid[:5]), 0.5, np.float32)])
        p5 = np.concatenate([parts, np.full(len(invalid[:5]), -1, np.int32)])
        got5, _ = oracle.train_ensemble(sp, E, H, idx5, t5, p5, w0, 15, 0.1, 0.5)
        assert np.array_equal(got5, ref)


def test_no_usable_sample_keeps_the_weights_and_single_network_uses_everything():
    sp, idx, t, parts, w0, E, H = small_problem(seed=10, n=40, E=2)
    P = sp.n_params
    per = H * P + 2 * H + 1
    got, loss = oracle.train_ensemble(sp, E, H, idx, np.full(len(idx), -1.0, np.float32), parts, w0, 5, 0.1, 0.0)
    assert np.array_equal(got, w0) and np.all(loss == 0.0)
    # one network, no sample in "part 0": trains on all the data
    none = np.full(len(idx), -1, np.int32)
    a, la = oracle.train_ensemble(sp, 1, H, idx, t, none, w0[:per], 10, 0.1, 0.0)
    use = usable_mask(sp, idx, t)
    x = np_features(sp, np_digits(sp, idx))[use]
    target = np.log(t[use].astype(np.float64))
    np.testing.assert_allclose(la[0, 0], np_loss(w0[:per], x, target, P, H), rtol=1e-12)
    np.testing.assert_allclose(la[0, -1], np_loss(a, x, target, P, H), rtol=1e-5)
    # plain gradient descent with a small step never increases the loss
    assert np.all(np.diff(la[0]) <= 1e-12)


# ---------------------------------------------------------------- metrics ----
def test_mean_relative_error_hand_values():
    pred = np.array([math.log(2.0), math.log(0.5), np.inf, math.log(3.0), 0.0], np.float32)
    times = np.array([1.0, 1.0, 1.0, -1.0, 4.0], np.float32)
    # |2-1|/1, |0.5-1|/1, (invalid skipped), (failed run skipped), |1-4|/4
    m, n = oracle.mean_relative_error(pred, times)
    assert n == 3
    assert abs(m - (1.0 + 0.5 + 0.75) / 3) < 1e-7
    assert oracle.mean_relative_error(np.array([np.inf], np.float32), np.array([1.0], np.float32)) == (0.0, 0)


def test_best_of_hand_values():
    assert oracle.best_of(np.array([3.0, 1.5, -1.0, 1.5, np.nan, 2.0], np.float32)) == (1, 1.5)
    pos, tm = oracle.best_of(np.array([-1.0, np.nan, 0.0, np.inf], np.float32))
    assert pos == -1 and math.isinf(tm)
    assert oracle.best_of(np.zeros(0, np.float32))[0] == -1
