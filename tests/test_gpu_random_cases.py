"""Seeded random cases: random spaces (irregular radices and rules, 2 to 23 parameters,
different spans of the fastest parameters), ensembles (one or two hidden layers of 1 to 128
units, 1 to 12 members), ranges, k and network evaluations.  Each case checks, against the CPU
oracle: mask bit for bit, predictions within the evaluation's tolerance, top-k by the band rule,
the list evaluation at the returned indices; and, inside the library: the selection against the
library's own predictions bit for bit, and the chunked / prepared / static-scratch calls against
the plain call bit for bit.  Run with -m gpu on an MI355X."""
import os

import numpy as np
import pytest

import oracle
import parity
import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)
TAILS = [(), (4, 3, 3), (2, 4, 4), (8, 4), (32,), (3, 16), (5, 7), (2, 2, 2, 2, 2)]
N_CASES = 320
BATCH = 40


def _nets():
    import paper_1506_00842_amd as T
    return {"f32": (dict(), parity.TOL_FP32),
            "split16": (dict(precision=T.TUNER_FP32, algo=T.TUNER_ALGO_SPLIT16), parity.TOL_FP32),
            "valu": (dict(precision=T.TUNER_FP32, algo=T.TUNER_ALGO_VALU), parity.TOL_FP32),
            "bf16": (dict(precision=T.TUNER_BF16_MFMA, algo=T.TUNER_ALGO_AUTO), 1e-2)}


def make_case(seed):
    rng = np.random.default_rng(seed)
    if rng.random() < 0.4:
        w = wl.random_small(seed, max_configs=int(rng.choice([64, 1024, 50000, 400000])),
                            n_hidden_layers=int(rng.choice([1, 2])), n_members=int(rng.integers(1, 13)),
                            hidden=int(rng.integers(1, 41)), n_constraints=int(rng.integers(0, 3)))
    else:
        P = int(rng.integers(2, 24))
        hidden = [int(rng.choice([1, 7, 16, 30, 32, 33, 64, 65, 100, 128])) for _ in range(int(rng.choice([1, 2])))]
        tail = TAILS[int(rng.integers(0, len(TAILS)))]
        if len(tail) >= P:
            tail = ()
        w = wl.many_params(P, hidden, int(rng.integers(1, 7)), seed=seed, pow2=bool(rng.random() < 0.5), tail=tail)
    n = w.space.n_configs
    widths = w.model.widths
    macs = sum(a * b for a, b in zip(widths[:-1], widths[1:])) * w.model.n_members
    count = int(min(n, max(1, int(3e9 / macs)), int(rng.choice([1, 37, 1000, 5000, 70000, 300000, 1200000]))))
    begin = int(rng.integers(0, n - count + 1))
    net = str(rng.choice(["f32", "split16", "valu", "bf16"]))
    k = int(rng.choice([1, 2, 10, 64, 100, 300, 512, 513, 1000, 3000]))
    return rng, w, begin, count, net, k


def run_case(seed):
    import paper_1506_00842_amd as T
    from paper_1506_00842_amd.api import Sweep
    rng, w, begin, count, net, k = make_case(seed)
    kw, tol = _nets()[net]
    sp, m = w.space, w.model
    print(f"case {seed}: {sp.name} N={sp.n_configs} widths={m.widths} E={m.n_members} net={net} k={k} "
          f"range=[{begin},+{count})", flush=True)
    oy, ov, _ = oracle.predict_range(sp, m, begin, count, threads=THREADS)
    sw = Sweep(sp, m, k, **kw)
    pred, mask = sw.predict_all(begin, count)
    torch.cuda.synchronize()
    assert np.array_equal(mask.cpu().numpy(), ov)
    parity.check_predictions(pred.cpu().numpy(), oy, ov, tol=tol)
    sw.topk(begin, count)
    torch.cuda.synchronize()
    gv, gi = sw.topk_host()
    parity.check_topk(gv, gi, oy, ov, begin, k, tol=tol)
    # the selection, against the library's own predictions
    gp = pred.cpu().numpy()
    valid_idx = np.nonzero(ov)[0]
    best = sorted(zip(gp[valid_idx].tolist(), (valid_idx + begin).tolist()))[:k]
    assert [x[1] for x in best] == gi.tolist()
    assert np.array_equal(np.array([x[0] for x in best], np.float32), gv)
    # the same range in pieces, in any order, with a running result; prepared or not
    cuts = sorted(set([0, count] + [int(c) for c in rng.integers(0, count + 1, int(rng.integers(1, 5)))]))
    order = list(range(len(cuts) - 1))
    rng.shuffle(order)
    sw2 = Sweep(sp, m, k, **kw)
    if rng.random() < 0.5:
        sw2.prepare()
    for j, piece in enumerate(order):
        sw2.topk(begin + cuts[piece], cuts[piece + 1] - cuts[piece], merge=j > 0)
    torch.cuda.synchronize()
    v2, i2 = sw2.topk_host()
    assert np.array_equal(i2, gi) and np.array_equal(v2, gv)
    sw2.prepare()
    p2, m2 = sw2.predict_all(begin, count)
    torch.cuda.synchronize()
    assert torch.equal(p2, pred) and torch.equal(m2, mask)
    # the call that allocates nothing
    if T.tuner_workspace_bytes(sw.space, sw.model, k) <= T.TUNER_STATIC_SCRATCH_BYTES:
        vals = torch.empty(k, dtype=torch.float32, device="cuda:0")
        idx = torch.empty(k, dtype=torch.int32, device="cuda:0")
        nf = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        T.tuner_predict_topk_static(sw.space, sw.model, begin, count, k, 0, vals, idx, nf, None)
        torch.cuda.synchronize()
        n_found = int(nf.item())
        assert n_found == len(gi)
        assert np.array_equal(idx[:n_found].cpu().numpy().view(np.uint32).astype(np.uint64), gi)
        assert np.array_equal(vals[:n_found].cpu().numpy(), gv)
    # the list evaluation at the returned indices
    if len(gi):
        it = torch.from_numpy(gi.astype(np.uint32).view(np.int32)).to("cuda:0")
        pi, mi = sw.predict_indices(it)
        torch.cuda.synchronize()
        ry, rv = oracle.predict_indices(sp, m, gi, threads=THREADS)
        assert rv.all() and mi.cpu().numpy().all()
        S = parity.scale_of(oy[ov.astype(bool)])
        err = np.abs(pi.cpu().numpy().astype(np.float64) - ry) / np.maximum(np.abs(ry), S)
        assert err.max() <= tol


@pytest.mark.parametrize("first", range(0, N_CASES, BATCH))
def test_random_cases(first):
    for seed in range(first, first + BATCH):
        run_case(seed)
