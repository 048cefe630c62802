"""Python binding of the MI355X full-space model sweep (argument marshalling only).

Every step of the path (decode, features, validity, ensemble evaluation, top-k)
runs in the HIP kernels of libtuner_hip.so; this module loads that library with
ctypes and converts tensors to pointers.  There is no CPU fallback: if the
library has not been built (python -m paper_1506_00842_amd.build) the import of
the entry points raises.

Function names and argument order follow include/tuner.h.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from .build import LIB_PATH

TUNER_OK = 0
TUNER_EINVAL, TUNER_ETOOLARGE, TUNER_ENOMEM, TUNER_EWORKSPACE, TUNER_EHIP = -1, -2, -3, -4, -5
TUNER_SCALE_LINEAR, TUNER_SCALE_LOG2 = 0, 1
TUNER_FP32, TUNER_BF16_MFMA = 0, 1
TUNER_ALGO_AUTO, TUNER_ALGO_MFMA, TUNER_ALGO_VALU, TUNER_ALGO_SPLIT16 = 0, 1, 2, 3
TUNER_MAX_K = 16384
TUNER_STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = [
    "tuner_space_create", "tuner_space_destroy", "tuner_space_size", "tuner_space_decode",
    "tuner_space_encode", "tuner_space_decode_device_arith", "tuner_workspace_bytes",
    "tuner_predict_topk", "tuner_predict_all", "tuner_decode_range", "tuner_last_error",
    "tuner_version", "tuner_profile_enable", "tuner_profile_read", "tuner_profile_read_train", "tuner_hoisted_parameters", "tuner_tabulated_parameters",
    "tuner_predict_indices", "tuner_sample_workspace_bytes", "tuner_sample_valid",
    "tuner_train_workspace_bytes", "tuner_train_ensemble", "tuner_mean_relative_error",
    "tuner_best_of", "tuner_predict_topk_static", "tuner_sweep_plan", "tuner_profile_pending", "tuner_prepare",
    "tuner_predict_topk_prepared", "tuner_predict_all_prepared",
]


class TunerError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"tuner error {code}: {msg}")
        self.code = code


class _TrainOptions(C.Structure):
    _fields_ = [("epochs", C.c_int32), ("learning_rate", C.c_float), ("momentum", C.c_float),
                ("workgroups_per_network", C.c_int32), ("barrier_poll_limit", C.c_int32)]


class _Model(C.Structure):
    _fields_ = [("n_members", C.c_int32), ("n_layers", C.c_int32),
                ("widths", C.POINTER(C.c_int32)), ("weights_dev", C.c_void_p),
                ("precision", C.c_int32), ("algo", C.c_int32)]


class _PlanInfo(C.Structure):
    _fields_ = [("network", C.c_int32), ("layer1", C.c_int32), ("waves", C.c_int32), ("tile", C.c_int32),
                ("variant_tiles_per_wave", C.c_int32), ("tiles_per_wave", C.c_int32), ("workgroups", C.c_int32),
                ("n_chunks", C.c_uint32), ("chunks_per_unit", C.c_int32), ("n_units", C.c_uint32),
                ("dynamic_queue", C.c_int32), ("live_chunk_list", C.c_int32), ("members_per_stage", C.c_int32),
                ("n_stages", C.c_int32), ("double_buffer", C.c_int32), ("pool_in_lds", C.c_int32),
                ("lds_bytes", C.c_int32), ("merge_launches", C.c_int32), ("workspace_bytes", C.c_size_t)]


_lib = None


def load_library():
    """Loads libtuner_hip.so (after torch, so that both share one HIP runtime)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with "
                          "`python -m paper_1506_00842_amd.build` (needs hipcc); "
                          "there is no fallback path")
    try:
        import torch  # noqa: F401  (loads the HIP runtime the library binds to)
    except ImportError:
        pass
    L = C.CDLL(LIB_PATH)
    L.tuner_last_error.restype = C.c_char_p
    L.tuner_version.restype = C.c_char_p
    L.tuner_workspace_bytes.restype = C.c_size_t
    L.tuner_space_destroy.restype = None
    L.tuner_space_create.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                     C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p)]
    L.tuner_space_destroy.argtypes = [C.c_void_p]
    L.tuner_hoisted_parameters.argtypes = [C.c_void_p, C.POINTER(_Model), C.POINTER(C.c_int32)]
    L.tuner_tabulated_parameters.argtypes = [C.c_void_p, C.POINTER(_Model), C.POINTER(C.c_int32)]
    L.tuner_space_size.argtypes = [C.c_void_p, C.POINTER(C.c_uint64)]
    L.tuner_space_decode.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.POINTER(C.c_int32)]
    L.tuner_space_decode_device_arith.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p,
                                                  C.POINTER(C.c_int32)]
    L.tuner_space_encode.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_uint64)]
    L.tuner_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(_Model), C.c_int32]
    L.tuner_predict_topk.argtypes = [C.c_void_p, C.POINTER(_Model), C.c_uint64, C.c_uint64,
                                     C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_size_t, C.c_void_p]
    L.tuner_sweep_plan.argtypes = [C.c_void_p, C.POINTER(_Model), C.c_uint64, C.c_uint64, C.c_int32,
                                   C.POINTER(_PlanInfo)]
    L.tuner_predict_topk_static.argtypes = [C.c_void_p, C.POINTER(_Model), C.c_uint64, C.c_uint64,
                                            C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p]
    L.tuner_predict_all.argtypes = [C.c_void_p, C.POINTER(_Model), C.c_uint64, C.c_uint64,
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.tuner_prepare.argtypes = [C.c_void_p, C.POINTER(_Model), C.c_void_p, C.c_size_t, C.c_void_p]
    L.tuner_predict_topk_prepared.argtypes = L.tuner_predict_topk.argtypes
    L.tuner_predict_all_prepared.argtypes = L.tuner_predict_all.argtypes
    L.tuner_decode_range.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p, C.c_void_p,
                                     C.c_void_p, C.c_void_p]
    L.tuner_predict_indices.argtypes = [C.c_void_p, C.POINTER(_Model), C.c_uint64, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.tuner_sample_workspace_bytes.restype = C.c_size_t
    L.tuner_sample_workspace_bytes.argtypes = [C.c_uint64]
    L.tuner_sample_valid.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint64, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.tuner_train_workspace_bytes.restype = C.c_size_t
    L.tuner_train_workspace_bytes.argtypes = [C.c_void_p, C.c_uint64]
    L.tuner_train_ensemble.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_uint64, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(_TrainOptions),
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.tuner_mean_relative_error.argtypes = [C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p,
                                            C.c_void_p, C.c_void_p]
    L.tuner_best_of.argtypes = [C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    _lib = L
    return L


def _check(rc: int):
    if rc != TUNER_OK:
        raise TunerError(rc, load_library().tuner_last_error().decode())


def tuner_last_error() -> str:
    return load_library().tuner_last_error().decode()


def tuner_hoisted_parameters(space, model) -> int:
    n = C.c_int32(0)
    _check(load_library().tuner_hoisted_parameters(space.ptr, C.byref(model.c), C.byref(n)))
    return int(n.value)


def tuner_tabulated_parameters(space, model) -> int:
    n = C.c_int32(0)
    _check(load_library().tuner_tabulated_parameters(space.ptr, C.byref(model.c), C.byref(n)))
    return int(n.value)


def tuner_sweep_plan(space, model, index_begin, index_count, k) -> dict:
    """What a sweep of this range would launch (host only), as a dict of the struct's fields."""
    info = _PlanInfo()
    _check(load_library().tuner_sweep_plan(space.ptr, C.byref(model.c), int(index_begin), int(index_count),
                                           int(k), C.byref(info)))
    return {name: int(getattr(info, name)) for name, _ in _PlanInfo._fields_}


def tuner_profile_enable(on: bool) -> None:
    _check(load_library().tuner_profile_enable(1 if on else 0))


def tuner_profile_pending() -> int:
    L = load_library()
    L.tuner_profile_pending.restype = C.c_int64
    return int(L.tuner_profile_pending())


def tuner_profile_read():
    """-> (summed sweep-kernel milliseconds, number of launches) since the last read."""
    ms = C.c_double(); n = C.c_int64()
    _check(load_library().tuner_profile_read(C.byref(ms), C.byref(n)))
    return float(ms.value), int(n.value)


def tuner_profile_read_train():
    """-> (summed training-kernel milliseconds, number of launches) since the last read."""
    ms = C.c_double(); n = C.c_int64()
    _check(load_library().tuner_profile_read_train(C.byref(ms), C.byref(n)))
    return float(ms.value), int(n.value)


def tuner_version() -> str:
    return load_library().tuner_version().decode()


class SpaceHandle:
    """Owns a tuner_space*; destroyed with the Python object."""

    def __init__(self, ptr: int, n_params: int):
        self.ptr = C.c_void_p(ptr)
        self.n_params = n_params

    def __del__(self):
        if getattr(self, "ptr", None) and _lib is not None:
            _lib.tuner_space_destroy(self.ptr)
            self.ptr = None


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def tuner_space_create(radices, values, scales, constraint_terms=None, constraint_bounds=None) -> SpaceHandle:
    L = load_library()
    rad = np.ascontiguousarray(radices, dtype=np.int32)
    vals = np.ascontiguousarray(values, dtype=np.float64)
    sc = np.ascontiguousarray(scales, dtype=np.int32)
    nc = 0 if constraint_bounds is None else len(constraint_bounds)
    terms = np.ascontiguousarray(constraint_terms, dtype=np.int32) if nc else None
    bounds = np.ascontiguousarray(constraint_bounds, dtype=np.int64) if nc else None
    out = C.c_void_p()
    _check(L.tuner_space_create(len(rad), _ptr(rad), _ptr(vals), _ptr(sc), nc, _ptr(terms),
                                _ptr(bounds), C.byref(out)))
    return SpaceHandle(out.value, len(rad))


def tuner_space_size(space: SpaceHandle) -> int:
    n = C.c_uint64()
    _check(load_library().tuner_space_size(space.ptr, C.byref(n)))
    return int(n.value)


def tuner_space_decode(space: SpaceHandle, index: int):
    """-> (digits i32[P], values f64[P], features f32[P], valid bool), host helper."""
    P = space.n_params
    d = np.empty(P, np.int32); v = np.empty(P, np.float64); f = np.empty(P, np.float32)
    ok = C.c_int32()
    _check(load_library().tuner_space_decode(space.ptr, index, _ptr(d), _ptr(v), _ptr(f), C.byref(ok)))
    return d, v, f, bool(ok.value)


def tuner_space_decode_device_arith(space: SpaceHandle, index: int):
    P = space.n_params
    d = np.empty(P, np.int32); f = np.empty(P, np.float32)
    ok = C.c_int32()
    _check(load_library().tuner_space_decode_device_arith(space.ptr, index, _ptr(d), _ptr(f), C.byref(ok)))
    return d, f, bool(ok.value)


def tuner_space_encode(space: SpaceHandle, digits) -> int:
    d = np.ascontiguousarray(digits, dtype=np.int32)
    out = C.c_uint64()
    _check(load_library().tuner_space_encode(space.ptr, _ptr(d), C.byref(out)))
    return int(out.value)


class ModelHandle:
    """tuner_model struct plus the arrays it points to (kept alive)."""

    def __init__(self, n_members: int, widths, weights_dev, precision=TUNER_FP32, algo=TUNER_ALGO_AUTO):
        self.widths = np.ascontiguousarray(widths, dtype=np.int32)
        self.weights_dev = weights_dev          # torch tensor on the GPU (fp32, contiguous)
        self.c = _Model(int(n_members), len(self.widths) - 1,
                        self.widths.ctypes.data_as(C.POINTER(C.c_int32)),
                        C.c_void_p(weights_dev.data_ptr() if hasattr(weights_dev, "data_ptr") else int(weights_dev)),
                        int(precision), int(algo))


def tuner_workspace_bytes(space: SpaceHandle, model: ModelHandle, k: int) -> int:
    n = load_library().tuner_workspace_bytes(space.ptr, C.byref(model.c), int(k))
    if n == 0:
        raise TunerError(TUNER_EINVAL, tuner_last_error())
    return int(n)


def _dp(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def tuner_predict_topk(space, model, index_begin, index_count, k, merge_with_existing,
                       topk_values_dev, topk_indices_dev, n_found_dev, workspace_dev, stream=None):
    _check(load_library().tuner_predict_topk(
        space.ptr, C.byref(model.c), int(index_begin), int(index_count), int(k),
        int(merge_with_existing), _dp(topk_values_dev), _dp(topk_indices_dev), _dp(n_found_dev),
        _dp(workspace_dev), workspace_dev.numel() * workspace_dev.element_size(), _stream(stream)))


def tuner_predict_topk_static(space, model, index_begin, index_count, k, merge_with_existing,
                              topk_values_dev, topk_indices_dev, n_found_dev, stream=None):
    _check(load_library().tuner_predict_topk_static(
        space.ptr, C.byref(model.c), int(index_begin), int(index_count), int(k),
        int(merge_with_existing), _dp(topk_values_dev), _dp(topk_indices_dev), _dp(n_found_dev),
        _stream(stream)))


def tuner_prepare(space, model, workspace_dev, stream=None):
    _check(load_library().tuner_prepare(space.ptr, C.byref(model.c), _dp(workspace_dev), _nbytes(workspace_dev),
                                        _stream(stream)))


def tuner_predict_topk_prepared(space, model, index_begin, index_count, k, merge_with_existing,
                                topk_values_dev, topk_indices_dev, n_found_dev, workspace_dev, stream=None):
    _check(load_library().tuner_predict_topk_prepared(
        space.ptr, C.byref(model.c), int(index_begin), int(index_count), int(k),
        int(merge_with_existing), _dp(topk_values_dev), _dp(topk_indices_dev), _dp(n_found_dev),
        _dp(workspace_dev), _nbytes(workspace_dev), _stream(stream)))


def tuner_predict_all_prepared(space, model, index_begin, index_count, predictions_dev, valid_mask_dev,
                               workspace_dev, stream=None):
    _check(load_library().tuner_predict_all_prepared(
        space.ptr, C.byref(model.c), int(index_begin), int(index_count), _dp(predictions_dev),
        _dp(valid_mask_dev), _dp(workspace_dev), _nbytes(workspace_dev), _stream(stream)))


def tuner_predict_all(space, model, index_begin, index_count, predictions_dev, valid_mask_dev,
                      workspace_dev, stream=None):
    _check(load_library().tuner_predict_all(
        space.ptr, C.byref(model.c), int(index_begin), int(index_count), _dp(predictions_dev),
        _dp(valid_mask_dev), _dp(workspace_dev),
        workspace_dev.numel() * workspace_dev.element_size(), _stream(stream)))


def tuner_decode_range(space, index_begin, index_count, digits_dev, features_dev, valid_mask_dev,
                       stream=None):
    _check(load_library().tuner_decode_range(
        space.ptr, int(index_begin), int(index_count), _dp(digits_dev), _dp(features_dev),
        _dp(valid_mask_dev), _stream(stream)))


def _nbytes(t):
    return t.numel() * t.element_size() if t is not None else 0


def tuner_predict_indices(space, model, n, indices_dev, predictions_dev, valid_mask_dev,
                          workspace_dev, stream=None):
    _check(load_library().tuner_predict_indices(
        space.ptr, C.byref(model.c), int(n), _dp(indices_dev), _dp(predictions_dev),
        _dp(valid_mask_dev), _dp(workspace_dev), _nbytes(workspace_dev), _stream(stream)))


def tuner_sample_workspace_bytes(max_draws: int) -> int:
    n = load_library().tuner_sample_workspace_bytes(int(max_draws))
    if n == 0:
        raise TunerError(TUNER_ETOOLARGE, tuner_last_error())
    return int(n)


def tuner_sample_valid(space, seed, n_samples, max_draws, indices_dev, n_found_dev, workspace_dev,
                       stream=None):
    _check(load_library().tuner_sample_valid(
        space.ptr, int(seed) & (2 ** 64 - 1), int(n_samples), int(max_draws), _dp(indices_dev),
        _dp(n_found_dev), _dp(workspace_dev), _nbytes(workspace_dev), _stream(stream)))


def tuner_train_workspace_bytes(space, n_samples: int) -> int:
    n = load_library().tuner_train_workspace_bytes(space.ptr, int(n_samples))
    if n == 0:
        raise TunerError(TUNER_ETOOLARGE, tuner_last_error())
    return int(n)


def tuner_train_ensemble(space, n_members, hidden, n_samples, sample_indices_dev, sample_times_dev,
                         sample_parts_dev, initial_weights_dev, epochs, learning_rate, momentum,
                         weights_out_dev, loss_history_dev, workspace_dev, stream=None,
                         workgroups_per_network=0, barrier_poll_limit=0):
    opt = _TrainOptions(int(epochs), float(learning_rate), float(momentum), int(workgroups_per_network),
                        int(barrier_poll_limit))
    _check(load_library().tuner_train_ensemble(
        space.ptr, int(n_members), int(hidden), int(n_samples), _dp(sample_indices_dev),
        _dp(sample_times_dev), _dp(sample_parts_dev), _dp(initial_weights_dev), C.byref(opt),
        _dp(weights_out_dev), _dp(loss_history_dev), _dp(workspace_dev), _nbytes(workspace_dev),
        _stream(stream)))


def tuner_mean_relative_error(n, predictions_dev, times_dev, mean_error_dev, n_used_dev, stream=None):
    _check(load_library().tuner_mean_relative_error(
        int(n), _dp(predictions_dev), _dp(times_dev), _dp(mean_error_dev), _dp(n_used_dev),
        _stream(stream)))


def tuner_best_of(m, times_dev, best_pos_dev, best_time_dev, stream=None):
    _check(load_library().tuner_best_of(int(m), _dp(times_dev), _dp(best_pos_dev), _dp(best_time_dev),
                                        _stream(stream)))
