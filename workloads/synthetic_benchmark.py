"""A synthetic stand-in for "compile and run the benchmark at configuration i".

The paper's tuner gets its training data and its second-stage measurements by
running OpenCL benchmarks (Sections 5.2 and 5.3); those kernels, devices and
measured times are not available, so this module produces seeded, repeatable
"execution times" with the character the paper describes: smooth dependence
on the parameters with interactions between them (work-group shape against
work per thread, memory-space flags), multiplicative measurement noise, and a
share of configurations that fail at run time although no static rule excludes
them (reported as a time of -1).

It is an input generator only: the times it returns are handed, as arrays, to
the CPU oracle and to the HIP library alike.  To know which parameter values a
configuration index stands for it uses numpy's unravel_index over the radices
(row-major, last parameter fastest), the same convention the oracle and the
library are each pinned to on their own.
"""
from __future__ import annotations

import numpy as np

from . import SCALE_LOG2, Space, Stream


class SyntheticBenchmark:
    """times(indices) -> float32 execution times in seconds (-1 = failed run)."""

    def __init__(self, space: Space, seed: int, noise_sigma: float = 0.03,
                 fail_fraction: float = 0.02):
        self.space = space
        self.seed = int(seed)
        self.noise_sigma = float(noise_sigma)
        self.fail_fraction = float(fail_fraction)
        P = space.n_params
        st = Stream(self.seed ^ 0xBE7C4)
        self.centre = 0.15 + 0.7 * st.uniform(P)              # best normalised value per parameter
        self.curv = 0.4 + 2.0 * st.uniform(P)                 # curvature per parameter
        self.pair = (st.uniform(P * P).reshape(P, P) - 0.5) * 1.2
        self.pair = np.triu(self.pair, 1)                     # pairwise interactions
        self.base = -6.0 + 2.0 * st.uniform(1)[0]             # ln(seconds) scale of the benchmark
        self._scaled = []
        for v, sc in zip(space.values, space.scales):
            t = np.log2(np.array(v, dtype=np.float64)) if sc == SCALE_LOG2 else np.array(v, dtype=np.float64)
            lo, hi = t.min(), t.max()
            self._scaled.append((t - lo) / (hi - lo) if hi > lo else np.zeros_like(t))

    def _unit_inputs(self, indices: np.ndarray) -> np.ndarray:
        idx = np.asarray(indices, dtype=np.int64)
        digs = np.unravel_index(idx, tuple(int(r) for r in self.space.radices))
        return np.stack([self._scaled[p][digs[p]] for p in range(self.space.n_params)], axis=1)

    def log_time_noise_free(self, indices) -> np.ndarray:
        u = self._unit_inputs(indices)
        d = u - self.centre
        quad = (self.curv * d * d).sum(axis=1)
        inter = np.einsum("np,pq,nq->n", d, self.pair, d)
        return self.base + quad + 0.5 * inter + 0.3 * np.sin(3.0 * u[:, 0] + 2.0 * u[:, 1])

    def times(self, indices) -> np.ndarray:
        idx = np.asarray(indices, dtype=np.uint64)
        lt = self.log_time_noise_free(idx)
        # per-configuration noise and failures from the counter-based generator at counter = index
        with np.errstate(over="ignore"):
            a = _hash64(idx, self.seed * 2 + 1)
            b = _hash64(idx, self.seed * 2 + 2)
            c = _hash64(idx, self.seed * 2 + 3)
        u1 = (a >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
        u2 = (b >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
        u3 = (c >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
        normal = np.sqrt(-2.0 * np.log(1.0 - u1)) * np.cos(2.0 * np.pi * u2)
        t = np.exp(lt + self.noise_sigma * normal)
        t[u3 < self.fail_fraction] = -1.0
        return t.astype(np.float32)


def _hash64(idx: np.ndarray, seed: int) -> np.ndarray:
    """splitmix64 output function of seed + (idx + 1) * gamma, vectorised."""
    z = np.uint64(seed & ((1 << 64) - 1)) + (idx + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15)
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def initial_weights(n_members: int, n_params: int, hidden: int, seed: int) -> np.ndarray:
    """Random initial weights for training (Section 4.2: training starts from random
    weights), layout W1[hidden][P], b1, w_o, b_o per network: W ~ N(0, 1/fan_in),
    b ~ U(-0.1, 0.1), fp32."""
    from . import make_model
    return make_model([n_params, hidden, 1], n_members, seed).weights


def parts_round_robin(n_samples: int, n_parts: int) -> np.ndarray:
    """Split of the training data into n_parts parts (Section 5.2, bagging): sample s
    belongs to part s mod n_parts (the samples are in random order already)."""
    return (np.arange(n_samples) % n_parts).astype(np.int32)
