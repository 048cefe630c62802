"""Seeded synthetic inputs for the full-space model sweep.

This module only *describes* problems: parameter value lists, scaling flags,
integer constraint tables, random ensemble weights and k.  It contains none of
the method's arithmetic (no index decoding, no feature normalisation, no network
evaluation, no selection); both the CPU oracle's tests and the HIP path's tests
draw their inputs from here so that the two sides see identical arrays.

Shapes follow the tuning spaces of the paper (Table 2: power-of-two work-group
and per-thread lists, boolean optimisation flags, small unroll lists) and the
model of Section 5.2 (bagged ensemble of small sigmoid networks); the measured
timings and trained weights of the paper are not available, so weights are
random draws from a documented counter-based generator.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

SCALE_LINEAR = 0
SCALE_LOG2 = 1

_MASK64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15


# --------------------------------------------------------------------------
# Counter-based uniform generator (splitmix64 output function applied to
# seed + (n+1)*gamma), vectorised over the counter n.
# --------------------------------------------------------------------------
def _splitmix64_block(seed: int, start: int, count: int) -> np.ndarray:
    n = np.arange(start + 1, start + count + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(seed & _MASK64) + n * np.uint64(_GAMMA)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return z


class Stream:
    """Sequential view of the counter-based generator."""

    def __init__(self, seed: int):
        self.seed = int(seed)
        self.pos = 0

    def uniform(self, count: int) -> np.ndarray:
        """count doubles in [0, 1): top 53 bits of each 64-bit word."""
        z = _splitmix64_block(self.seed, self.pos, count)
        self.pos += count
        return (z >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)

    def normal(self, count: int) -> np.ndarray:
        """count standard normals; each uses two consecutive uniforms (u1, u2):
        sqrt(-2 ln(1-u1)) * cos(2 pi u2)."""
        u = self.uniform(2 * count)
        u1 = u[0::2]
        u2 = u[1::2]
        return np.sqrt(-2.0 * np.log(1.0 - u1)) * np.cos(2.0 * math.pi * u2)

    def integers(self, count: int, high: int) -> np.ndarray:
        """count integers in [0, high) (high <= 2**53)."""
        return np.minimum((self.uniform(count) * high).astype(np.uint64), np.uint64(high - 1))


# --------------------------------------------------------------------------
# Problem descriptions
# --------------------------------------------------------------------------
@dataclass
class Space:
    """Cartesian-product tuning space: one value list per parameter
    (Section 5.1, Table 2), a per-parameter scaling flag for the network input,
    and statically known validity rules in separable integer form: a
    configuration with digits d is valid iff, for every rule c,
    sum_p terms[c][offset_p + d_p] <= bounds[c]."""

    name: str
    values: List[List[float]]
    scales: List[int]
    constraint_terms: np.ndarray = field(default_factory=lambda: np.zeros((0, 0), np.int32))
    constraint_bounds: np.ndarray = field(default_factory=lambda: np.zeros((0,), np.int64))
    param_names: List[str] = field(default_factory=list)

    @property
    def n_params(self) -> int:
        return len(self.values)

    @property
    def radices(self) -> np.ndarray:
        return np.array([len(v) for v in self.values], dtype=np.int32)

    @property
    def flat_values(self) -> np.ndarray:
        return np.array([x for v in self.values for x in v], dtype=np.float64)

    @property
    def offsets(self) -> np.ndarray:
        r = self.radices
        return np.concatenate([[0], np.cumsum(r)[:-1]]).astype(np.int64)

    @property
    def n_configs(self) -> int:
        n = 1
        for v in self.values:
            n *= len(v)
        return n

    @property
    def n_constraints(self) -> int:
        return int(self.constraint_bounds.shape[0])

    def without_constraints(self) -> "Space":
        return Space(self.name + "-unconstrained", self.values, self.scales,
                     np.zeros((0, int(self.radices.sum())), np.int32),
                     np.zeros((0,), np.int64), self.param_names)


@dataclass
class Model:
    """Bagged ensemble (Section 5.2): n_members networks with identical layer
    widths [P, H1, (H2,) 1]; hidden layers use the logistic sigmoid, the output
    is linear.  `weights` is one fp32 array: per member, per dense layer,
    W[out][in] row-major followed by b[out]."""

    widths: List[int]
    n_members: int
    weights: np.ndarray
    seed: int = -1

    @property
    def floats_per_member(self) -> int:
        return sum(self.widths[l] * self.widths[l + 1] + self.widths[l + 1]
                   for l in range(len(self.widths) - 1))

    @property
    def macs_per_config(self) -> int:
        return self.n_members * sum(self.widths[l] * self.widths[l + 1]
                                    for l in range(len(self.widths) - 1))

    @property
    def sigmoids_per_config(self) -> int:
        return self.n_members * sum(self.widths[1:-1])

    def member_layers(self, e: int):
        """[(W[out,in], b[out]), ...] views for member e (no arithmetic)."""
        off = e * self.floats_per_member
        out = []
        for l in range(len(self.widths) - 1):
            fi, fo = self.widths[l], self.widths[l + 1]
            W = self.weights[off:off + fi * fo].reshape(fo, fi)
            off += fi * fo
            b = self.weights[off:off + fo]
            off += fo
            out.append((W, b))
        return out


@dataclass
class Workload:
    name: str
    space: Space
    model: Model
    k: int
    chunk: int = 0          # index-range chunk size for streamed sweeps (0 = whole space)
    n_valid: int = -1       # analytic count of valid configurations (-1: not stated)
    note: str = ""


def make_model(widths: Sequence[int], n_members: int, seed: int) -> Model:
    """W ~ N(0, 1/fan_in), b ~ U(-0.1, 0.1); draw order member -> layer ->
    W row-major -> b; values rounded to fp32."""
    st = Stream(seed)
    parts = []
    for _e in range(n_members):
        for l in range(len(widths) - 1):
            fi, fo = widths[l], widths[l + 1]
            W = st.normal(fi * fo) / math.sqrt(fi)
            b = -0.1 + 0.2 * st.uniform(fo)
            parts.append(W)
            parts.append(b)
    w = np.concatenate(parts).astype(np.float32)
    return Model(list(widths), n_members, w, seed)


def _pow2(n: int) -> List[float]:
    return [float(1 << j) for j in range(n)]


def _terms(space_values: List[List[float]], per_param: dict) -> np.ndarray:
    """One constraint row: per_param maps parameter index -> list of integer
    terms (one per value of that parameter); other parameters contribute 0."""
    row = []
    for p, v in enumerate(space_values):
        t = per_param.get(p)
        if t is None:
            row.extend([0] * len(v))
        else:
            assert len(t) == len(v)
            row.extend(int(x) for x in t)
    return np.array(row, dtype=np.int32)


def _log2_terms(vals: Sequence[float]) -> List[int]:
    out = []
    for v in vals:
        e = int(round(math.log2(v)))
        assert float(1 << e) == v
        out.append(e)
    return out


# ---- the five benchmark workloads -----------------------------------------
def tiny() -> Workload:
    """256 configurations, all valid; one 4-16-1 network, seed 0, k = 10."""
    values = [_pow2(4), _pow2(4), [0.0, 1.0], [float(v) for v in range(1, 9)]]
    scales = [SCALE_LOG2, SCALE_LOG2, SCALE_LINEAR, SCALE_LINEAR]
    sp = Space("tiny", values, scales,
               np.zeros((0, 18), np.int32), np.zeros((0,), np.int64),
               ["a", "b", "flag", "c"])
    return Workload("cfg1-tiny", sp, make_model([4, 16, 1], 1, 0), 10, n_valid=256)


def conv_shaped() -> Workload:
    """Convolution-shaped space: 393,216 configurations, valid iff
    wg_x * wg_y <= 1024; 8 networks 10-30-1, seed 1, k = 100."""
    values = [_pow2(8), _pow2(8),
              [float(v) for v in range(1, 9)], [float(v) for v in range(1, 9)],
              [0.0, 1.0], [0.0, 1.0], [0.0, 1.0], [0.0, 1.0], [0.0, 1.0],
              [0.0, 1.0, 2.0]]
    scales = [SCALE_LOG2, SCALE_LOG2] + [SCALE_LINEAR] * 8
    names = ["wg_x", "wg_y", "ept_x", "ept_y", "unroll", "local", "image",
             "padding", "interleave", "filter_cache"]
    t = _terms(values, {0: _log2_terms(values[0]), 1: _log2_terms(values[1])})
    sp = Space("conv-shaped", values, scales, t[None, :], np.array([10], np.int64), names)
    return Workload("cfg2-conv", sp, make_model([10, 30, 1], 8, 1), 100, n_valid=331_776)


def _large_space(radices: Sequence[int], name: str) -> Space:
    values, scales = [], []
    for r in radices:
        if r == 8:
            values.append(_pow2(8)); scales.append(SCALE_LOG2)
        elif r == 4:
            values.append(_pow2(4)); scales.append(SCALE_LOG2)
        elif r == 2:
            values.append([0.0, 1.0]); scales.append(SCALE_LINEAR)
        else:
            raise ValueError(r)
    c0 = _terms(values, {0: _log2_terms(values[0]), 1: _log2_terms(values[1])})
    # "third value <= fourth value": both lists are identical and increasing,
    # so this is digit_2 - digit_3 <= 0.
    c1 = _terms(values, {2: list(range(len(values[2]))),
                         3: [-j for j in range(len(values[3]))]})
    return Space(name, values, scales, np.stack([c0, c1]), np.array([10, 0], np.int64))


LARGE_RADICES = [8, 8, 8, 8, 4, 4, 4, 4, 4, 2, 2, 2, 2, 2]          # product 2**27
LARGE_RADICES_AS_WRITTEN = [8, 8, 8, 8, 4, 4, 4, 4, 2, 2, 2, 2, 2, 2]  # product 2**26


def large() -> Workload:
    """2**27 configurations, 14 parameters; 4 networks 14-64-64-1, seed 2, k = 1000."""
    sp = _large_space(LARGE_RADICES, "large-2^27")
    return Workload("cfg3-large", sp, make_model([14, 64, 64, 1], 4, 2), 1000,
                    n_valid=63_700_992)


def large_as_written() -> Workload:
    """Labelled extra: the 14-radix list whose product is 2**26."""
    sp = _large_space(LARGE_RADICES_AS_WRITTEN, "large-2^26")
    return Workload("cfg3-2^26", sp, make_model([14, 64, 64, 1], 4, 2), 1000,
                    n_valid=31_850_496)


def wide() -> Workload:
    """Same space as large(); 16 networks 14-128-128-1, seed 3, k = 1000."""
    sp = _large_space(LARGE_RADICES, "large-2^27")
    return Workload("cfg4-wide", sp, make_model([14, 128, 128, 1], 16, 3), 1000,
                    n_valid=63_700_992)


STREAMED_RADICES = [16, 16, 16, 4, 4, 4] + [2] * 14                   # product 2**32


def streamed() -> Workload:
    """2**32 configurations, 20 parameters, swept in 2**28-index chunks with a
    running top-4096; 8 networks 20-64-64-1, seed 4.  Three linear rules leave
    3,011,788,800 configurations valid (29.9 % invalid)."""
    values, scales = [], []
    for r in STREAMED_RADICES:
        if r == 16:
            values.append([float(v) for v in range(1, 17)]); scales.append(SCALE_LOG2)
        elif r == 4:
            values.append(_pow2(4)); scales.append(SCALE_LOG2)
        else:
            values.append([0.0, 1.0]); scales.append(SCALE_LINEAR)
    fx = [int(round((1 << 20) * math.log2(v))) for v in values[0]]
    c0 = _terms(values, {0: fx, 1: fx, 2: fx})                     # v0*v1*v2 <= 1024
    c1 = _terms(values, {3: _log2_terms(values[3]), 4: _log2_terms(values[4]),
                         5: _log2_terms(values[5])})               # log2 sum <= 7
    c2 = _terms(values, {6: [0, 1], 7: [0, 1], 8: [0, 1], 9: [0, 1]})  # at most 3 of 4 flags
    sp = Space("streamed-2^32", values, scales, np.stack([c0, c1, c2]),
               np.array([10 << 20, 7, 3], np.int64))
    return Workload("cfg5-streamed", sp, make_model([20, 64, 64, 1], 8, 4), 4096,
                    chunk=1 << 28, n_valid=3_011_788_800)


# ---- the paper's own spaces (Table 2) with its 11 x (P-30-1) ensemble -------
def _paper_space(name: str, extra: List[List[float]], extra_scales: List[int],
                 extra_names: List[str]) -> Space:
    common = [_pow2(8), _pow2(8), _pow2(8), _pow2(8)]
    values = common + extra
    scales = [SCALE_LOG2] * 4 + extra_scales
    names = ["wg_x", "wg_y", "ppt_x", "ppt_y"] + extra_names
    # statically known rule used here: work-group size wg_x * wg_y <= 1024
    # (a typical device limit; Section 5.2 names work-group limits as a cause
    # of invalid configurations)
    t = _terms(values, {0: _log2_terms(values[0]), 1: _log2_terms(values[1])})
    return Space(name, values, scales, t[None, :], np.array([10], np.int64), names)


def paper_convolution(seed: int = 11, k: int = 200) -> Workload:
    sp = _paper_space("convolution", [[0.0, 1.0]] * 5, [SCALE_LINEAR] * 5,
                      ["image", "local", "padding", "interleave", "unroll"])
    return Workload("paper-convolution", sp, make_model([9, 30, 1], 11, seed), k, n_valid=110_592)


def paper_raycasting(seed: int = 12, k: int = 300) -> Workload:
    sp = _paper_space("raycasting", [[0.0, 1.0]] * 5 + [[1.0, 2.0, 4.0, 8.0, 16.0]],
                      [SCALE_LINEAR] * 5 + [SCALE_LOG2],
                      ["image_data", "image_tf", "local_tf", "const_tf", "interleave", "unroll"])
    return Workload("paper-raycasting", sp, make_model([10, 30, 1], 11, seed), k, n_valid=552_960)


def paper_stereo(seed: int = 13, k: int = 300) -> Workload:
    sp = _paper_space("stereo", [[0.0, 1.0]] * 4 + [_pow2(4), _pow2(3), _pow2(3)],
                      [SCALE_LINEAR] * 4 + [SCALE_LOG2] * 3,
                      ["image_l", "image_r", "local_l", "local_r", "unroll_disp",
                       "unroll_dx", "unroll_dy"])
    return Workload("paper-stereo", sp, make_model([11, 30, 1], 11, seed), k, n_valid=1_990_656)


# ---- small irregular spaces for brute-force tests --------------------------
def random_small(seed: int, max_configs: int = 1024, n_hidden_layers: int = 1,
                 n_members: int = 3, hidden: int = 7, k: int = 17,
                 n_constraints: int = 2) -> Workload:
    """Irregular space (radices 1..6, non-power-of-two values, mixed scaling,
    random small integer rules) with at most max_configs configurations."""
    st = Stream(seed ^ 0xABCDEF)
    values, scales = [], []
    n = 1
    while True:
        r = int(st.integers(1, 6)[0]) + 1
        if n * r > max_configs or len(values) >= 8:
            break
        lo = float(int(st.integers(1, 5)[0]) + 1)
        step = float(int(st.integers(1, 3)[0]) + 1)
        vals = [lo + step * j for j in range(r)]
        values.append(vals)
        scales.append(int(st.integers(1, 2)[0]))
        n *= r
    if not values:
        values, scales = [[1.0, 2.0, 3.0]], [SCALE_LINEAR]
    total = sum(len(v) for v in values)
    terms = np.zeros((n_constraints, total), np.int32)
    bounds = np.zeros((n_constraints,), np.int64)
    for c in range(n_constraints):
        terms[c] = st.integers(total, 7).astype(np.int64) - 3
        # keep roughly the lower two thirds of the reachable sums
        bounds[c] = int(st.integers(1, 4)[0]) + 1
    sp = Space(f"random-small-{seed}", values, scales, terms, bounds)
    widths = [len(values)] + [hidden] * n_hidden_layers + [1]
    return Workload(sp.name, sp, make_model(widths, n_members, seed), k)


def many_params(n_params: int, widths_hidden: Sequence[int], n_members: int, seed: int,
                k: int = 50, pow2: bool = False, tail: Sequence[int] = ()) -> Workload:
    """A space with many parameters (radices 3, 5, 2, 2, ... or all 2) to reach
    the wider input paddings of the kernels; one random small-integer rule.
    `tail` replaces the radices of the last parameters (how many configurations the
    fastest parameters span decides how the sweep evaluates layer 1)."""
    radices = [2] * n_params
    if n_params > 29:
        pow2 = True           # 45 * 2**(P-3) would exceed 2**32
    radices[n_params - len(tail):] = list(tail)
    if not pow2:
        radices[0] = 3
        if n_params > 1:
            radices[1] = 5
        if n_params > 4:
            radices[4] = 3
    values = [[float(j + 1) for j in range(r)] for r in radices]
    scales = [SCALE_LOG2 if p % 3 == 0 else SCALE_LINEAR for p in range(n_params)]
    st = Stream(seed ^ 0x5EED)
    total = sum(radices)
    terms = (st.integers(total, 5).astype(np.int64) - 2).astype(np.int32)[None, :]
    bounds = np.array([n_params // 3], np.int64)
    sp = Space(f"many-{n_params}-{'pow2' if pow2 else 'mixed'}{'-tail' + 'x'.join(map(str, tail)) if tail else ''}",
               values, scales, terms, bounds)
    return Workload(sp.name, sp, make_model([n_params, *widths_hidden, 1], n_members, seed), k)


def large_with_members(n_members: int) -> Workload:
    """The 2**27 space with a different ensemble size (kernel studies)."""
    sp = _large_space(LARGE_RADICES, "large-2^27")
    return Workload(f"cfg3-E{n_members}", sp, make_model([14, 64, 64, 1], n_members, 2), 1000,
                    n_valid=63_700_992)


def large_unconstrained() -> Workload:
    """The 2**27 space without validity rules (the paper's own sweep masks nothing)."""
    w = large()
    sp = w.space
    free = Space("large-2^27-unconstrained", sp.values, sp.scales)
    return Workload("cfg3-unconstrained", free, w.model, w.k, n_valid=free.n_configs)


BENCH_WORKLOADS = {
    "cfg3-E1": lambda: large_with_members(1), "cfg3-E8": lambda: large_with_members(8),
    "cfg1": tiny, "cfg2": conv_shaped, "cfg3": large, "cfg4": wide, "cfg5": streamed,
    "cfg3-2^26": large_as_written, "cfg3-unconstrained": lambda: large_unconstrained(),
    "paper-convolution": paper_convolution, "paper-raycasting": paper_raycasting,
    "paper-stereo": paper_stereo,
}
