"""GPU parity tests for the stages around the sweep: random choice of valid
training configurations, ensemble evaluation at a list of configurations,
training of the bagged ensemble, mean relative error and the second-stage
pick — the HIP library (through the C ABI) against the CPU oracle on the same
seeded inputs.  Integer results (sample indices, positions, counts) are
compared bit for bit.  Run with -m gpu on an MI355X.

Tolerances of the fp32 training against the fp64 oracle:
  * loss at the initial weights and the first update: the loss is a mean of n
    squares computed from ~1-ulp sigmoids and fp32 sums of n terms; the error of
    a sum of n fp32 terms added in a tree of per-lane chains is a few n^(1/2)
    ulp in practice and at most n ulp, so 1e-5 relative covers n <= 4000 with a
    wide margin; the gradient (read back as (w0 - w1) / eta) is checked against
    the largest gradient entry at 2e-5;
  * whole trajectories: rounding differences are carried through the momentum
    recursion and amplified by 1 / (1 - mu) and by the curvature of the loss, so
    the loss history is checked at 1e-4 relative and the weights at 2e-4 of the
    largest weight, for runs of at most 200 epochs (observed: below 3e-6 and 1e-6).
"""
import os

import numpy as np
import pytest

import oracle
import parity
import workloads as wl
from workloads.synthetic_benchmark import SyntheticBenchmark, initial_weights, parts_round_robin

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)


def say(*a):
    print(*a, flush=True)


def tuner_for(space):
    from paper_1506_00842_amd.api import Tuner
    return Tuner(space)


def dev_u32(a):
    return torch.from_numpy(np.ascontiguousarray(a).astype(np.uint32).view(np.int32)).cuda()


def host_u32(t):
    return t.cpu().numpy().view(np.uint32)


# ---------------------------------------------------------------- sampler ----
SAMPLER_CASES = [
    (wl.tiny, 1, 40, 200), (wl.conv_shaped, 2, 500, 900), (wl.paper_stereo, 3, 300, 400),
    (wl.paper_convolution, 7, 4000, 1 << 13), (wl.large, 5, 3000, 1 << 14),
    (wl.streamed, 0xFEDCBA9876543210, 64, 4096), (wl.streamed, 11, 50000, 1 << 17),
    (lambda: wl.random_small(5, n_constraints=2), 4, 50, 5000),
    (lambda: wl.random_small(9, n_constraints=2), 5, 10_000, 30_000),     # space smaller than n
    (wl.paper_raycasting, 9, 1, 1), (wl.paper_raycasting, 10, 100_000, 1 << 20),
]


@pytest.mark.parametrize("maker,seed,n,max_draws", SAMPLER_CASES)
def test_sampler_bit_exact(maker, seed, n, max_draws):
    sp = maker().space
    say("sampler", sp.name, seed, n, max_draws)
    tn = tuner_for(sp)
    idx, found = tn.sample_valid(seed, n, max_draws)
    torch.cuda.synchronize()
    expect = oracle.sample_valid(sp, seed, n, max_draws)
    got = host_u32(idx)
    nf = int(found.item())
    assert nf == len(expect)
    assert np.array_equal(got[:nf].astype(np.uint64), expect)
    assert np.all(got[nf:] == 0xFFFFFFFF)


def test_sampler_errors():
    from paper_1506_00842_amd import TunerError
    tn = tuner_for(wl.tiny().space)
    with pytest.raises(TunerError):
        tn.sample_valid(1, 10, 5)            # max_draws < n_samples
    with pytest.raises(TunerError):
        tn.sample_valid(1, 0, 5)
    with pytest.raises(TunerError):
        tn.sample_valid(1, 10, (1 << 24) + 1)


# -------------------------------------------------------- predict_indices ----
@pytest.mark.parametrize("maker,n", [
    (wl.tiny, 1), (wl.conv_shaped, 33), (wl.paper_convolution, 1000), (wl.paper_stereo, 70001),
    (wl.large, 20011), (wl.streamed, 4097),
])
def test_predict_indices_matches_oracle(maker, n):
    from paper_1506_00842_amd.api import Sweep
    w = maker()
    sp = w.space
    say("predict_indices", w.name, n)
    rng = np.random.default_rng(n)
    idx = rng.integers(0, sp.n_configs, size=n, dtype=np.uint64)
    idx[0] = sp.n_configs - 1
    sw = Sweep(sp, w.model, 0)
    pred, mask = sw.predict_indices(dev_u32(idx))
    torch.cuda.synchronize()
    oy, ov = oracle.predict_indices(sp, w.model, idx, threads=THREADS)
    assert np.array_equal(mask.cpu().numpy(), ov)
    worst, rel = parity.check_predictions(pred.cpu().numpy(), oy, ov)
    say(f"  worst {worst:.3f} x tol, pure-relative worst {rel:.2e}")
    # the same configurations through the range entry point: same values up to the order of
    # the fp32 additions (a range sweep may take the layer-1 share of the parameters that are
    # constant over a tile out of the matrix instructions; a list cannot)
    lo = int(idx[-1])
    cnt = int(min(64, sp.n_configs - lo))
    a, ma = sw.predict_all(lo, cnt)
    b, mb = sw.predict_indices(dev_u32(np.arange(lo, lo + cnt, dtype=np.uint64)))
    torch.cuda.synchronize()
    assert torch.equal(ma, mb)
    va, vb = a[ma.bool()], b[mb.bool()]
    assert bool(torch.all(torch.abs(va - vb) <= 2e-6 * torch.clamp(torch.abs(va), min=1.0)))


# --------------------------------------------------------------- training ----
def problem(maker, seed, n, E, H, fail_fraction=0.05):
    w = maker()
    sp = w.space
    idx = oracle.sample_valid(sp, seed, n, 64 * n)
    bm = SyntheticBenchmark(sp, seed, fail_fraction=fail_fraction)
    t = bm.times(idx)
    # a single network has no part to leave out: it trains on all the data
    parts = parts_round_robin(len(idx), E) if E > 1 else np.full(len(idx), -1, np.int32)
    w0 = initial_weights(E, sp.n_params, H, seed + 100)
    return sp, idx, t, parts, w0


def gpu_train(sp, E, H, idx, t, parts, w0, epochs, eta, mu, **kw):
    tn = tuner_for(sp)
    w, loss = tn.train(E, H, idx, t, parts, w0, epochs, eta, mu, **kw)
    torch.cuda.synchronize()
    return w.cpu().numpy(), loss.cpu().numpy()


TRAIN_CASES = [  # maker, seed, n, E, H, epochs, eta, mu
    (lambda: wl.random_small(3, max_configs=600, n_constraints=1), 3, 60, 3, 4, 40, 0.0625, 0.875),
    (wl.tiny, 1, 100, 1, 1, 30, 0.125, 0.5),
    (wl.paper_convolution, 21, 2000, 11, 30, 120, 0.125, 0.875),          # the paper's shape (Section 5.2)
    (wl.paper_stereo, 22, 777, 11, 30, 60, 0.125, 0.75),
    (wl.conv_shaped, 23, 1000, 4, 32, 50, 0.125, 0.5),
    (wl.conv_shaped, 24, 513, 3, 33, 50, 0.125, 0.5),                     # 64-lane groups, padded units
    (wl.streamed, 25, 1500, 8, 64, 40, 0.0625, 0.75),                     # 20 inputs, 64 units
    (lambda: wl.many_params(25, [8], 1, 3), 26, 300, 2, 17, 40, 0.0625, 0.5),
    (wl.large, 27, 4000, 2, 30, 200, 0.125, 0.875),
    (lambda: wl.many_params(31, [8], 1, 3), 28, 400, 3, 64, 30, 0.0625, 0.5),   # widest kernel: 31 inputs, 64 units
    (lambda: wl.many_params(31, [8], 1, 3), 29, 900, 2, 20, 30, 0.0625, 0.5),
]


@pytest.mark.parametrize("maker,seed,n,E,H,epochs,eta,mu", TRAIN_CASES)
def test_training_matches_oracle(maker, seed, n, E, H, epochs, eta, mu):
    sp, idx, t, parts, w0 = problem(maker, seed, n, E, H)
    say("train", sp.name, "n", len(idx), "E", E, "H", H, "epochs", epochs)
    P = sp.n_params
    per = H * P + 2 * H + 1
    # first update only: loss at the initial weights and the gradient
    g1, gl1 = gpu_train(sp, E, H, idx, t, parts, w0, 1, eta, 0.0)
    o1, ol1 = oracle.train_ensemble(sp, E, H, idx, t, parts, w0, 1, eta, 0.0)
    np.testing.assert_allclose(gl1, ol1, rtol=1e-5)
    for e in range(E):
        gg = (w0[e * per:(e + 1) * per].astype(np.float64) - g1[e * per:(e + 1) * per]) / eta
        og = (w0[e * per:(e + 1) * per].astype(np.float64) - o1[e * per:(e + 1) * per]) / eta
        scale = max(np.abs(og).max(), 1.0)
        assert np.abs(gg - og).max() <= 2e-5 * scale
    # the whole run
    gw, gl = gpu_train(sp, E, H, idx, t, parts, w0, epochs, eta, mu)
    ow, ol = oracle.train_ensemble(sp, E, H, idx, t, parts, w0, epochs, eta, mu)
    worst_l = np.max(np.abs(gl - ol) / ol)
    worst_w = np.abs(gw - ow).max() / np.abs(ow).max()
    say(f"  loss {ol[:, 0].mean():.4f} -> {ol[:, -1].mean():.4f}; worst loss rel {worst_l:.2e}, weights {worst_w:.2e}")
    assert worst_l <= 1e-4
    assert worst_w <= 2e-4
    assert np.all(ol[:, -1] < ol[:, 0])
    # reproducible bit for bit
    gw2, gl2 = gpu_train(sp, E, H, idx, t, parts, w0, epochs, eta, mu)
    assert np.array_equal(gw, gw2) and np.array_equal(gl, gl2)


@pytest.mark.parametrize("split", [1, 2, 3, 7, 16])
def test_training_any_number_of_workgroups_per_network(split):
    """The samples of a network are split over several workgroups that exchange partial
    sums once per epoch: every split must meet the same tolerances (only the order of the
    fp32 additions differs), ragged slices included (777 samples over 7 workgroups)."""
    sp, idx, t, parts, w0 = problem(wl.paper_stereo, 51, 777, 5, 30)
    E, H, epochs, eta, mu = 5, 30, 80, 0.125, 0.75
    ow, ol = oracle.train_ensemble(sp, E, H, idx, t, parts, w0, epochs, eta, mu)
    gw, gl = gpu_train(sp, E, H, idx, t, parts, w0, epochs, eta, mu, workgroups_per_network=split)
    worst_l = np.max(np.abs(gl - ol) / ol)
    worst_w = np.abs(gw - ow).max() / np.abs(ow).max()
    say(f"  split {split}: worst loss rel {worst_l:.2e}, weights {worst_w:.2e}")
    assert worst_l <= 1e-4 and worst_w <= 2e-4
    gw2, gl2 = gpu_train(sp, E, H, idx, t, parts, w0, epochs, eta, mu, workgroups_per_network=split)
    assert np.array_equal(gw, gw2) and np.array_equal(gl, gl2)


def test_training_long_run_is_reproducible_and_learns():
    """3000 epochs of the paper-shaped problem, twice: 176 workgroups meet 3001 times per
    run; any stale read in the exchange of partial sums would show as a difference."""
    sp, idx, t, parts, w0 = problem(wl.paper_convolution, 61, 2000, 11, 30)
    a_w, a_l = gpu_train(sp, 11, 30, idx, t, parts, w0, 3000, 0.125, 0.875)
    b_w, b_l = gpu_train(sp, 11, 30, idx, t, parts, w0, 3000, 0.125, 0.875)
    assert np.all(np.isfinite(a_w)) and np.all(np.isfinite(a_l))
    assert np.array_equal(a_w, b_w) and np.array_equal(a_l, b_l)
    assert np.all(a_l[:, -1] < 0.02 * a_l[:, 0])
    # the last loss is the loss of the returned weights: check it with the oracle's forward pass
    _, ol = oracle.train_ensemble(sp, 11, 30, idx, t, parts, a_w, 0, 0.125, 0.875)
    np.testing.assert_allclose(a_l[:, -1], ol[:, 0], rtol=1e-4)


def test_training_gives_up_cleanly_when_the_barrier_times_out():
    """A poll limit of 1 makes workgroups give up as soon as they have to wait: the kernel
    must still end, and every network is either complete (bit-identical to a normal run)
    or all NaN, never a partial result."""
    sp, idx, t, parts, w0 = problem(wl.paper_convolution, 62, 2000, 11, 30)
    E, H, epochs = 11, 30, 200
    per = H * sp.n_params + 2 * H + 1
    ref_w, ref_l = gpu_train(sp, E, H, idx, t, parts, w0, epochs, 0.125, 0.875)
    got_w, got_l = gpu_train(sp, E, H, idx, t, parts, w0, epochs, 0.125, 0.875, barrier_poll_limit=1)
    n_nan = 0
    for e in range(E):
        we, le = got_w[e * per:(e + 1) * per], got_l[e]
        if np.isnan(we).any() or np.isnan(le).any():
            assert np.isnan(we).all() and np.isnan(le).all()
            n_nan += 1
        else:
            assert np.array_equal(we, ref_w[e * per:(e + 1) * per]) and np.array_equal(le, ref_l[e])
    say(f"  {n_nan} of {E} networks gave up with a poll limit of 1")
    # and the library is usable afterwards
    again_w, again_l = gpu_train(sp, E, H, idx, t, parts, w0, epochs, 0.125, 0.875)
    assert np.array_equal(again_w, ref_w) and np.array_equal(again_l, ref_l)


def test_training_edge_cases():
    sp, idx, t, parts, w0 = problem(wl.conv_shaped, 31, 200, 3, 8, fail_fraction=0.2)
    E, H = 3, 8
    # no epochs: weights returned unchanged, one loss value per network
    gw, gl = gpu_train(sp, E, H, idx, t, parts, w0, 0, 0.1, 0.5)
    _, ol = oracle.train_ensemble(sp, E, H, idx, t, parts, w0, 0, 0.1, 0.5)
    assert np.array_equal(gw, w0)
    np.testing.assert_allclose(gl, ol, rtol=1e-5)
    # every run failed: nothing to train on
    bad = np.full(len(idx), -1.0, np.float32)
    gw, gl = gpu_train(sp, E, H, idx, bad, parts, w0, 5, 0.1, 0.5)
    assert np.array_equal(gw, w0) and np.all(gl == 0.0)
    # failed runs written as -1, 0, NaN, inf and invalid configurations are all ignored alike
    t2 = t.copy()
    failed = np.nonzero(~(t > 0))[0]
    assert len(failed) >= 4
    for n_, b in enumerate(failed):
        t2[b] = [-1.0, 0.0, np.nan, np.inf][n_ % 4]
    ref_w, ref_l = gpu_train(sp, E, H, idx, t, parts, w0, 20, 0.1, 0.5)
    got_w, got_l = gpu_train(sp, E, H, idx, t2, parts, w0, 20, 0.1, 0.5)
    assert np.array_equal(ref_w, got_w) and np.array_equal(ref_l, got_l)
    _, ov, _ = oracle.predict_range(sp, None, 0, sp.n_configs, threads=THREADS, want_yhat=False)
    invalid = np.nonzero(ov == 0)[0][:7].astype(np.uint64)
    idx3 = np.concatenate([idx, invalid])
    t3 = np.concatenate([t, np.full(len(invalid), 0.5, np.float32)])
    p3 = np.concatenate([parts, np.full(len(invalid), -1, np.int32)])
    ow, ol = oracle.train_ensemble(sp, E, H, idx3, t3, p3, w0, 20, 0.1, 0.5)
    gw3, gl3 = gpu_train(sp, E, H, idx3, t3, p3, w0, 20, 0.1, 0.5)
    np.testing.assert_allclose(gl3, ol, rtol=1e-4)
    np.testing.assert_allclose(gl3, ref_l, rtol=1e-6)      # only the summation order may differ
    # network e never sees part e: changing that part's times leaves it unchanged bit for bit
    t4 = t.copy()
    t4[parts == 1] *= 3.0
    w4, _ = gpu_train(sp, E, H, idx, t4, parts, w0, 20, 0.1, 0.5)
    per = H * sp.n_params + 2 * H + 1
    assert np.array_equal(w4[per:2 * per], ref_w[per:2 * per])
    assert not np.array_equal(w4[:per], ref_w[:per])


def test_training_in_place_and_errors():
    from paper_1506_00842_amd import (TunerError, tuner_train_ensemble, tuner_train_workspace_bytes)
    sp, idx, t, parts, w0 = problem(wl.tiny, 41, 50, 2, 6)
    tn = tuner_for(sp)
    ref, _ = tn.train(2, 6, idx, t, parts, w0, 10, 0.1, 0.5)
    n = len(idx)
    ws = torch.empty(tuner_train_workspace_bytes(tn.space, n), dtype=torch.uint8, device="cuda")
    w = torch.from_numpy(w0).cuda()
    args = (dev_u32(idx), torch.from_numpy(t).cuda(), torch.from_numpy(parts).cuda())
    tuner_train_ensemble(tn.space, 2, 6, n, *args, w, 10, 0.1, 0.5, w, None, ws)   # output aliases input, no loss
    torch.cuda.synchronize()
    assert torch.equal(w, ref)
    with pytest.raises(TunerError):
        tuner_train_ensemble(tn.space, 2, 65, n, *args, w, 10, 0.1, 0.5, w, None, ws)
    with pytest.raises(TunerError):
        tuner_train_ensemble(tn.space, 0, 6, n, *args, w, 10, 0.1, 0.5, w, None, ws)
    with pytest.raises(TunerError):
        tuner_train_ensemble(tn.space, 2, 6, n, *args, w, -1, 0.1, 0.5, w, None, ws)
    with pytest.raises(TunerError):
        tuner_train_ensemble(tn.space, 2, 6, n, *args, w, 10, 0.1, 0.5, w, None, ws[:256])


# ---------------------------------------------------------------- metrics ----
def test_mean_relative_error_and_best_of():
    tn = tuner_for(wl.tiny().space)
    rng = np.random.default_rng(5)
    for n in (0, 1, 5, 1023, 1024, 1025, 100_003):
        pred = rng.normal(-5.0, 1.0, n).astype(np.float32)
        times = np.exp(rng.normal(-5.0, 1.0, n)).astype(np.float32)
        if n >= 5:
            pred[1] = np.inf                       # an invalid configuration
            times[2] = -1.0                        # failed runs
            times[3] = np.nan
            times[4] = 0.0
        m, cnt = tn.mean_relative_error(torch.from_numpy(pred).cuda(), torch.from_numpy(times).cuda())
        pos, bt = tn.best_of(torch.from_numpy(times).cuda())
        torch.cuda.synchronize()
        om, on = oracle.mean_relative_error(pred, times)
        assert int(cnt.item()) == on
        assert abs(float(m.item()) - om) <= 1e-5 * max(om, 1e-30)
        opos, obt = oracle.best_of(times)
        assert int(pos.item()) == opos
        assert float(bt.item()) == obt or (opos == -1 and np.isinf(float(bt.item())))
    # ties go to the earliest entry; all failed -> -1
    tt = np.array([3.0, 1.5, -1.0, 1.5, np.nan, 2.0] * 400, np.float32)
    pos, bt = tn.best_of(torch.from_numpy(tt).cuda())
    assert (int(pos.item()), float(bt.item())) == (1, 1.5)
    pos, bt = tn.best_of(torch.from_numpy(np.array([-1.0, np.nan, 0.0, np.inf], np.float32)).cuda())
    assert int(pos.item()) == -1 and np.isinf(float(bt.item()))


# ------------------------------------------------------------- whole tuner ---
def test_two_stage_tuner_end_to_end():
    """Section 5 on the convolution space with the paper's settings (N = 2000 training
    configurations, 11 networks of 30 units, M = 200), every stage on the GPU with a
    synthetic benchmark in place of the OpenCL runs; the same pipeline through the
    oracle selects from the same candidates."""
    from paper_1506_00842_amd.api import Sweep
    w = wl.paper_convolution()
    sp = w.space
    P, E, H, N_train, M = sp.n_params, 11, 30, 2000, 200
    bm = SyntheticBenchmark(sp, 77)
    tn = tuner_for(sp)
    idx_dev, found = tn.sample_valid(77, N_train, 8 * N_train)
    assert int(found.item()) == N_train
    idx = host_u32(idx_dev).astype(np.uint64)
    assert np.array_equal(idx, oracle.sample_valid(sp, 77, N_train, 8 * N_train))
    t = bm.times(idx)
    parts = parts_round_robin(N_train, E)
    w0 = initial_weights(E, P, H, 770)
    epochs, eta, mu = 200, 0.125, 0.875
    gw, gl = tn.train(E, H, idx_dev, t, parts, w0, epochs, eta, mu)
    ow, ol = oracle.train_ensemble(sp, E, H, idx, t, parts, w0, epochs, eta, mu)
    np.testing.assert_allclose(gl.cpu().numpy(), ol, rtol=1e-4)
    # accuracy on configurations not used for training (Section 6)
    held = np.setdiff1d(oracle.sample_valid(sp, 78, 1500, 12000), idx)[:1000]
    t_held = bm.times(held)
    model = wl.Model([P, H, 1], E, gw.cpu().numpy())
    sw = Sweep(sp, model, M)
    pred, _ = sw.predict_indices(dev_u32(held))
    err, used = tn.mean_relative_error(pred, torch.from_numpy(t_held).cuda())
    o_pred, _ = oracle.predict_indices(sp, wl.Model([P, H, 1], E, ow), held, threads=THREADS)
    o_err, o_used = oracle.mean_relative_error(o_pred, t_held)
    say(f"  mean relative error on {int(used.item())} held-out configurations: gpu {float(err.item()):.4f}, oracle {o_err:.4f}")
    assert int(used.item()) == o_used
    assert abs(float(err.item()) - o_err) <= 2e-3
    assert o_err < 0.5
    # first stage: the M lowest predictions; second stage: the best of their measured times
    sw.topk(0, sp.n_configs)
    gv, gi = sw.topk_host()
    oy, ov, _ = oracle.predict_range(sp, model, 0, sp.n_configs, threads=THREADS)
    parity.check_topk(gv, gi, oy, ov, 0, M)
    t_cand = bm.times(gi.astype(np.uint64))
    pos, bt = tn.best_of(torch.from_numpy(t_cand).cuda())
    opos, obt = oracle.best_of(t_cand)
    assert int(pos.item()) == opos and float(bt.item()) == obt
    all_t = bm.times(np.arange(sp.n_configs, dtype=np.uint64))
    best_valid = all_t[(ov == 1) & (all_t > 0)].min()
    say(f"  tuner result {obt:.3e} s vs global optimum {best_valid:.3e} s: slowdown {obt / best_valid:.3f}")
    assert obt / best_valid < 1.5


def test_tune_function_runs_the_whole_tuner():
    """api.tune on the stereo space (2,359,296 configurations) with the settings the paper
    uses for its large spaces (3000 training configurations, M = 300)."""
    from paper_1506_00842_amd.api import tune
    sp = wl.paper_stereo().space
    bm = SyntheticBenchmark(sp, 91)
    calls = []

    def measure(indices):
        calls.append(len(indices))
        return bm.times(indices)

    res = tune(sp, measure, initial_weights(11, sp.n_params, 30, 910), n_train=3000, m=300, epochs=300, seed=91)
    assert calls == [3000, 300]
    assert res["best_index"] is not None and np.all(np.isfinite(res["final_loss"]))
    assert res["best_time"] == np.min(res["candidate_times"][res["candidate_times"] > 0])
    # against the best of 50,000 random valid configurations (the paper's yardstick for the
    # spaces it could not search exhaustively)
    ref = bm.times(oracle.sample_valid(sp, 92, 50_000, 400_000))
    best_random = ref[ref > 0].min()
    say(f"  tuner {res['best_time']:.4e} s vs best of 50,000 random {best_random:.4e} s: ratio {res['best_time'] / best_random:.3f}")
    assert res["best_time"] < 1.25 * best_random
