"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Loads oracle/liboracle.so (built by oracle/build.py with g++) and marshals
arguments; every computation happens in tuner_oracle.cpp.  Only tests, the
smoke check and the benchmark's cpu_baseline leg may import this package; the
HIP library and its Python binding never do.

The `space` and `model` arguments are duck-typed: a space needs
radices / flat_values / scales / constraint_terms / constraint_bounds, a model
needs n_members / widths / weights (fp32).
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from .build import LIB_PATH, build

_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            build()
        L = C.CDLL(LIB_PATH)
        L.oracle_select_topk.restype = C.c_int64
        L.oracle_sample_valid.restype = C.c_int64
        L.oracle_mean_relative_error.restype = C.c_double
        L.oracle_best_of.restype = C.c_int64
        _lib = L
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t)) if a is not None else None


def _space_args(space):
    rad = np.ascontiguousarray(space.radices, dtype=np.int32)
    vals = np.ascontiguousarray(space.flat_values, dtype=np.float64)
    sc = np.ascontiguousarray(space.scales, dtype=np.int32)
    terms = np.ascontiguousarray(space.constraint_terms, dtype=np.int32)
    bounds = np.ascontiguousarray(space.constraint_bounds, dtype=np.int64)
    keep = (rad, vals, sc, terms, bounds)
    return keep, (C.c_int(len(rad)), _p(rad, C.c_int32), _p(vals, C.c_double), _p(sc, C.c_int32),
                  C.c_int(len(bounds)), _p(terms, C.c_int32), _p(bounds, C.c_int64))


def feature_lut(space) -> np.ndarray:
    keep, a = _space_args(space)
    out = np.empty(int(keep[0].sum()), np.float32)
    lib().oracle_feature_lut(a[0], a[1], a[2], a[3], _p(out, C.c_float))
    return out


def digits(space, index: int) -> np.ndarray:
    rad = np.ascontiguousarray(space.radices, dtype=np.int32)
    out = np.empty(len(rad), np.int32)
    lib().oracle_digits(C.c_int(len(rad)), _p(rad, C.c_int32), C.c_uint64(index), _p(out, C.c_int32))
    return out


def index(space, digs) -> int:
    rad = np.ascontiguousarray(space.radices, dtype=np.int32)
    d = np.ascontiguousarray(digs, dtype=np.int32)
    out = C.c_uint64(0)
    lib().oracle_index(C.c_int(len(rad)), _p(rad, C.c_int32), _p(d, C.c_int32), C.byref(out))
    return int(out.value)


def predict_range(space, model, begin: int, count: int, threads: int = 1,
                  want_yhat: bool = True, want_digits: bool = False):
    """Returns (yhat fp32[count] or None, valid u8[count], digits i32[count,P] or None)."""
    keep, a = _space_args(space)
    P = len(keep[0])
    yhat = np.empty(count, np.float32) if want_yhat else None
    valid = np.empty(count, np.uint8)
    digs = np.empty((count, P), np.int32) if want_digits else None
    if model is not None:
        widths = np.ascontiguousarray(model.widths, dtype=np.int32)
        w = np.ascontiguousarray(model.weights, dtype=np.float32)
        nm, nl = int(model.n_members), len(widths) - 1
        assert widths[0] == P and widths[-1] == 1
    else:
        assert not want_yhat
        widths = np.zeros(1, np.int32); w = np.zeros(1, np.float32); nm, nl = 0, 0
    lib().oracle_predict_range(*a, C.c_int(nm), C.c_int(nl), _p(widths, C.c_int32),
                               _p(w, C.c_float), C.c_uint64(begin), C.c_uint64(count),
                               _p(yhat, C.c_float), _p(valid, C.c_uint8), _p(digs, C.c_int32),
                               C.c_int(threads))
    return yhat, valid, digs


def predict_indices(space, model, indices, threads: int = 1):
    """Returns (yhat fp32[n], valid u8[n]) for an arbitrary list of indices."""
    keep, a = _space_args(space)
    idx = np.ascontiguousarray(indices, dtype=np.uint64)
    yhat = np.empty(len(idx), np.float32)
    valid = np.empty(len(idx), np.uint8)
    widths = np.ascontiguousarray(model.widths, dtype=np.int32)
    w = np.ascontiguousarray(model.weights, dtype=np.float32)
    lib().oracle_predict_indices(*a, C.c_int(int(model.n_members)), C.c_int(len(widths) - 1),
                                 _p(widths, C.c_int32), _p(w, C.c_float), _p(idx, C.c_uint64),
                                 C.c_uint64(len(idx)), _p(yhat, C.c_float), _p(valid, C.c_uint8),
                                 C.c_int(threads))
    return yhat, valid


def select_topk(yhat, valid, index_base: int, k: int):
    """k smallest (value, index) among valid entries, ascending."""
    yhat = np.ascontiguousarray(yhat, dtype=np.float32)
    v = np.ascontiguousarray(valid, dtype=np.uint8) if valid is not None else None
    vals = np.empty(max(k, 1), np.float32)
    idx = np.empty(max(k, 1), np.uint64)
    n = lib().oracle_select_topk(_p(yhat, C.c_float), _p(v, C.c_uint8), C.c_uint64(len(yhat)),
                                 C.c_uint64(index_base), C.c_int64(k), _p(vals, C.c_float),
                                 _p(idx, C.c_uint64))
    return vals[:n].copy(), idx[:n].copy()


def topk(space, model, begin: int, count: int, k: int, threads: int = 1):
    yhat, valid, _ = predict_range(space, model, begin, count, threads)
    return select_topk(yhat, valid, begin, k)


def sample_valid(space, seed: int, n_samples: int, max_draws: int) -> np.ndarray:
    """First n_samples distinct valid indices in draw order (uint64)."""
    keep, a = _space_args(space)
    out = np.empty(max(n_samples, 1), np.uint64)
    n = lib().oracle_sample_valid(a[0], a[1], a[4], a[5], a[6], C.c_uint64(seed & (2 ** 64 - 1)),
                                  C.c_int64(n_samples), C.c_uint64(max_draws), _p(out, C.c_uint64))
    return out[:n].copy()


def train_ensemble(space, n_members: int, hidden: int, indices, times, parts, initial_weights,
                   epochs: int, learning_rate: float, momentum: float):
    """Returns (weights fp32[E * per], loss float64[E, epochs + 1])."""
    keep, a = _space_args(space)
    idx = np.ascontiguousarray(indices, dtype=np.uint64)
    t = np.ascontiguousarray(times, dtype=np.float32)
    pt = np.ascontiguousarray(parts, dtype=np.int32)
    w0 = np.ascontiguousarray(initial_weights, dtype=np.float32)
    P = len(keep[0])
    per = hidden * P + hidden + hidden + 1
    assert len(w0) == n_members * per and len(t) == len(idx) == len(pt)
    w = np.empty_like(w0)
    loss = np.empty((n_members, epochs + 1), np.float64)
    lib().oracle_train_ensemble(*a, C.c_int(n_members), C.c_int(hidden), C.c_int64(len(idx)),
                                _p(idx, C.c_uint64), _p(t, C.c_float), _p(pt, C.c_int32),
                                _p(w0, C.c_float), C.c_int(epochs), C.c_float(learning_rate),
                                C.c_float(momentum), _p(w, C.c_float), _p(loss, C.c_double))
    return w, loss


def mean_relative_error(predictions, times):
    """(mean of |exp(prediction) - t| / t over usable entries, count)."""
    p = np.ascontiguousarray(predictions, dtype=np.float32)
    t = np.ascontiguousarray(times, dtype=np.float32)
    n = C.c_int64(0)
    m = lib().oracle_mean_relative_error(C.c_int64(len(p)), _p(p, C.c_float), _p(t, C.c_float), C.byref(n))
    return float(m), int(n.value)


def best_of(times):
    """(position of the lowest usable time or -1, that time)."""
    t = np.ascontiguousarray(times, dtype=np.float32)
    bt = C.c_float(0)
    pos = lib().oracle_best_of(C.c_int64(len(t)), _p(t, C.c_float), C.byref(bt))
    return int(pos), float(bt.value)
