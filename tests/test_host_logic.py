"""CPU tests of the HIP library's host side: the C ABI loads and exports every
declared symbol, argument validation, space tables, and the device decoder's
arithmetic evaluated on the host (no kernel is launched here)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import workloads as wl
import paper_1506_00842_amd as T

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def make_space(sp):
    return T.tuner_space_create(sp.radices, sp.flat_values, sp.scales, sp.constraint_terms,
                                sp.constraint_bounds)


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "tuner.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(tuner_[a-z_0-9]+)\s*\(", hdr))
    assert {"tuner_space_create", "tuner_predict_topk", "tuner_predict_all"} <= names
    L = T.load_library()
    for n in sorted(names):
        assert hasattr(L, n), f"{n} declared in tuner.h but not exported"
    assert set(T.EXPORTS) == names
    assert "gfx950" in T.tuner_version()


def test_space_size_and_limits():
    for maker, n in ((wl.tiny, 256), (wl.conv_shaped, 393216), (wl.large, 1 << 27),
                     (wl.streamed, 1 << 32), (wl.paper_stereo, 2359296)):
        assert T.tuner_space_size(make_space(maker().space)) == n
    with pytest.raises(T.TunerError) as e:                     # 2^33 configurations
        T.tuner_space_create([2] * 31 + [4], [0.0, 1.0] * 31 + [1.0, 2.0, 3.0, 4.0], [0] * 32)
    assert e.value.code == T.TUNER_ETOOLARGE
    with pytest.raises(T.TunerError) as e:                     # exactly 2^32 + something
        T.tuner_space_create([65536, 65537], list(range(65536 + 65537)), [0, 0])
    assert e.value.code == T.TUNER_ETOOLARGE
    with pytest.raises(T.TunerError) as e:
        T.tuner_space_create([2, 0], [0.0, 1.0], [0, 0])
    assert e.value.code == T.TUNER_EINVAL
    with pytest.raises(T.TunerError) as e:
        T.tuner_space_create([2], [0.0, 1.0], [1])             # log2(0)
    assert e.value.code == T.TUNER_EINVAL
    with pytest.raises(T.TunerError) as e:
        T.tuner_space_create([2], [1.0, 2.0], [7])             # bad scale flag
    assert e.value.code == T.TUNER_EINVAL
    with pytest.raises(T.TunerError) as e:
        T.tuner_space_create([2], [1.0, float("nan")], [0])
    assert e.value.code == T.TUNER_EINVAL
    with pytest.raises(T.TunerError) as e:                     # rule sum overflows int32
        T.tuner_space_create([2, 2], [0, 1, 0, 1], [0, 0],
                             np.array([[2**31 - 1, 0, 2**31 - 1, 0]], np.int32), [0])
    assert e.value.code == T.TUNER_EINVAL
    with pytest.raises(T.TunerError) as e:
        T.tuner_space_create([300], list(range(300)), [0])
    assert e.value.code == T.TUNER_ETOOLARGE
    assert "too many values" in T.tuner_last_error()


def _irregular_spaces():
    yield wl.Space("odd", [[1.0, 2.0, 3.0], [5.0], [1.0, 2.0, 4.0, 8.0, 16.0], [0.0, 1.0],
                           [float(v) for v in range(1, 8)], [3.0, 9.0, 27.0]],
                   [0, 1, 1, 0, 0, 1],
                   np.array([[0, 1, 2, 0, 0, 1, 2, 3, 4, 0, 0] + [0] * 7 + [0, 0, 0],
                             [0] * 11 + [-3, -2, -1, 0, 1, 2, 3] + [5, 0, -5]], np.int32),
                   np.array([4, 1], np.int64))
    yield wl.Space("big-radices", [[float(v) for v in range(1, 251)], [1.0], [1.0, 2.0]],
                   [1, 0, 0])
    yield wl.Space("single", [[float(v) for v in range(1, 98)]], [0])
    for maker in (wl.paper_raycasting, wl.paper_stereo, wl.conv_shaped, wl.large, wl.streamed):
        yield maker().space
    for seed in (1, 2, 3, 4, 5, 6, 7):
        yield wl.random_small(seed).space


@pytest.mark.parametrize("sp", list(_irregular_spaces()), ids=lambda s: s.name)
def test_device_decoder_arithmetic_matches_oracle(sp):
    """digits, fp32 features and validity computed with the kernels' own
    multiply-shift routine (on the host) == the oracle's plain division."""
    h = make_space(sp)
    n = sp.n_configs
    st = wl.Stream(99)
    idx = [0, 1, n - 1, n // 2] + [int(v) for v in st.integers(1500, n)]
    if n <= 4096:
        idx = list(range(n))
    lut = oracle.feature_lut(sp)
    off = sp.offsets
    for i in idx:
        _, ov, od = oracle.predict_range(sp, None, i, 1, want_yhat=False, want_digits=True)
        d1, vals, f1, ok1 = T.tuner_space_decode(h, i)
        d2, f2, ok2 = T.tuner_space_decode_device_arith(h, i)
        assert np.array_equal(d1, od[0]) and np.array_equal(d2, od[0])
        assert ok1 == bool(ov[0]) and ok2 == bool(ov[0])
        expect_f = np.array([lut[off[p] + od[0][p]] for p in range(sp.n_params)], np.float32)
        assert np.array_equal(f1, expect_f) and np.array_equal(f2, expect_f)
        assert list(vals) == [sp.values[p][od[0][p]] for p in range(sp.n_params)]
        assert T.tuner_space_encode(h, d1) == i


def test_decode_encode_errors():
    h = make_space(wl.tiny().space)
    with pytest.raises(T.TunerError):
        T.tuner_space_decode(h, 256)
    with pytest.raises(T.TunerError):
        T.tuner_space_encode(h, [0, 0, 2, 0])
    with pytest.raises(T.TunerError):
        T.tuner_space_encode(h, [0, -1, 0, 0])


def test_bounds_outside_int32_are_clamped_not_wrapped():
    vals = [[0.0, 1.0], [0.0, 1.0]]
    terms = np.array([[0, 1, 0, 1], [0, 1, 0, 1]], np.int32)
    sp = wl.Space("clamp", vals, [0, 0], terms, np.array([2**40, -2**40], np.int64))
    h = make_space(sp)
    for i in range(4):
        assert T.tuner_space_decode(h, i)[3] is False              # second rule can never hold
        assert T.tuner_space_decode_device_arith(h, i)[2] is False
    sp2 = wl.Space("clamp2", vals, [0, 0], terms[:1], np.array([2**40], np.int64))
    h2 = make_space(sp2)
    assert all(T.tuner_space_decode_device_arith(h2, i)[2] for i in range(4))


class _FakeWeights:
    """Stands in for a device tensor where no kernel will be launched."""

    def data_ptr(self):
        return 0x1000


def test_workspace_bytes_and_model_validation():
    w = wl.large()
    h = make_space(w.space)
    m = T.ModelHandle(w.model.n_members, w.model.widths, _FakeWeights())
    b0 = T.tuner_workspace_bytes(h, m, 0)
    b1 = T.tuner_workspace_bytes(h, m, 1000)
    b2 = T.tuner_workspace_bytes(h, m, 4096)
    assert 0 < b0 < b1 < b2 and b0 % 256 == 0
    for bad, code in (
        (T.ModelHandle(4, [13, 64, 64, 1], _FakeWeights()), None),        # input width != P
        (T.ModelHandle(4, [14, 64, 64, 2], _FakeWeights()), None),        # output width != 1
        (T.ModelHandle(4, [14, 64, 64, 64, 1], _FakeWeights()), None),    # too deep
        (T.ModelHandle(0, [14, 64, 1], _FakeWeights()), None),            # no members
        (T.ModelHandle(4, [14, 300, 1], _FakeWeights()), None),           # too wide
        (T.ModelHandle(4, [14, 64, 1], _FakeWeights(), precision=7), None),                 # unknown precision
        (T.ModelHandle(4, [14, 64, 1], _FakeWeights(), algo=9), None),                      # unknown algo
        (T.ModelHandle(4, [14, 64, 1], _FakeWeights(), precision=T.TUNER_BF16_MFMA,
                       algo=T.TUNER_ALGO_SPLIT16), None),                                   # bf16 is MFMA only
    ):
        with pytest.raises(T.TunerError):
            T.tuner_workspace_bytes(h, bad, 10)
    with pytest.raises(T.TunerError):
        T.tuner_workspace_bytes(h, m, T.TUNER_MAX_K + 1)
    # every network evaluation has a workspace size
    for kw in (dict(algo=T.TUNER_ALGO_SPLIT16), dict(precision=T.TUNER_BF16_MFMA)):
        assert T.tuner_workspace_bytes(h, T.ModelHandle(4, [14, 64, 64, 1], _FakeWeights(), **kw), 1000) > 0


def test_predict_argument_errors_before_any_gpu_work():
    """Invalid calls are rejected on the host (no HIP call is reached)."""
    L = T.load_library()
    w = wl.tiny()
    h = make_space(w.space)
    m = T.ModelHandle(1, w.model.widths, _FakeWeights())
    fake = C.c_void_p(0x2000)
    # null outputs
    assert L.tuner_predict_topk(h.ptr, C.byref(m.c), 0, 256, 10, 0, None, fake, fake, fake, 1 << 30, None) == T.TUNER_EINVAL
    # k out of range
    assert L.tuner_predict_topk(h.ptr, C.byref(m.c), 0, 256, 0, 0, fake, fake, fake, fake, 1 << 30, None) == T.TUNER_EINVAL
    assert L.tuner_predict_topk(h.ptr, C.byref(m.c), 0, 256, T.TUNER_MAX_K + 1, 0, fake, fake, fake, fake, 1 << 30, None) == T.TUNER_ETOOLARGE
    # range outside the space
    assert L.tuner_predict_topk(h.ptr, C.byref(m.c), 200, 57, 10, 0, fake, fake, fake, fake, 1 << 30, None) == T.TUNER_EINVAL
    assert L.tuner_predict_all(h.ptr, C.byref(m.c), 257, 0, fake, None, fake, 1 << 30, None) == T.TUNER_EINVAL
    # workspace missing / too small / misaligned
    need = T.tuner_workspace_bytes(h, m, 10)
    assert L.tuner_predict_topk(h.ptr, C.byref(m.c), 0, 256, 10, 0, fake, fake, fake, None, need, None) == T.TUNER_EWORKSPACE
    assert L.tuner_predict_topk(h.ptr, C.byref(m.c), 0, 256, 10, 0, fake, fake, fake, fake, need - 1, None) == T.TUNER_EWORKSPACE
    assert L.tuner_predict_topk(h.ptr, C.byref(m.c), 0, 256, 10, 0, fake, fake, fake, C.c_void_p(0x2010), need, None) == T.TUNER_EWORKSPACE
    assert "workspace" in T.tuner_last_error()
    assert L.tuner_decode_range(h.ptr, 0, 257, None, None, None, None) == T.TUNER_EINVAL
    assert L.tuner_decode_range(None, 0, 1, None, None, None, None) == T.TUNER_EINVAL


def test_sweep_plan_of_the_benchmark_configurations():
    """How the library would cut a sweep into chunks and launches (no GPU here: the plan uses
    MI355X's 256 compute units and 160 KB of LDS)."""
    def plan(w, begin, count, k, **kw):
        h = make_space(w.space)
        return T.tuner_sweep_plan(h, T.ModelHandle(w.model.n_members, w.model.widths, _FakeWeights(), **kw),
                                  begin, count, k)
    w = wl.large()
    p = plan(w, 0, 1 << 27, 1000)
    assert p["network"] == 0 and p["layer1"] == 2 and p["waves"] == 16 and p["tile"] == 32
    assert p["tiles_per_wave"] == p["variant_tiles_per_wave"] == 2
    assert p["workgroups"] == 256 and p["n_chunks"] == (1 << 27) // 1024
    assert p["dynamic_queue"] == 1 and p["live_chunk_list"] == 1
    assert p["n_stages"] == 1 and p["members_per_stage"] == 4 and p["pool_in_lds"] == 1
    assert p["lds_bytes"] <= 160 * 1024 - 64
    assert p["workspace_bytes"] <= T.tuner_workspace_bytes(
        make_space(w.space), T.ModelHandle(4, w.model.widths, _FakeWeights()), 1000)
    p = plan(w, 0, 1 << 27, 0)                       # predict_all: no merge, no pool
    assert p["merge_launches"] == 0 and p["pool_in_lds"] == 0
    # the wide network streams one member at a time through two LDS buffers
    ww = wl.wide()
    p = plan(ww, 0, 1 << 27, 1000)
    assert p["layer1"] == 1 and p["waves"] == 8 and p["members_per_stage"] == 1 and p["n_stages"] == 16
    assert p["double_buffer"] == 1 and p["pool_in_lds"] == 0
    # bf16, 128 wide: 16 waves per workgroup, chunks of 1024 configurations (two tiles per wave)
    # for calls of 2^21 configurations or more; shorter calls take whichever of one or two
    # tiles per wave gives fewer rounds of chunks over the 256 workgroups
    for count, r in ((1 << 27, 2), ((1 << 21) + 777, 2), ((1 << 18) - 5, 2), ((1 << 18) + 777, 1), (1 << 14, 1), (1 << 13, 1), (12007, 1)):
        p = plan(ww, 0 if count == 1 << 27 else 3 << 18, count, 0, precision=T.TUNER_BF16_MFMA)
        assert p["network"] == 1 and p["waves"] == 16 and p["variant_tiles_per_wave"] == 2, (count, p)
        assert p["tiles_per_wave"] == r, (count, p)
    assert p["members_per_stage"] == 2 and p["double_buffer"] == 1
    # the streamed space: chunks of 2^28, two members per stage
    ws = wl.streamed()
    p = plan(ws, 5 << 28, 1 << 28, 4096)
    assert p["layer1"] == 2 and p["members_per_stage"] == 2 and p["n_stages"] == 4 and p["double_buffer"] == 1
    assert p["live_chunk_list"] == 1
    # a short sweep (the paper's convolution space): one chunk per workgroup, no queue, no list
    wc = wl.paper_convolution()
    p = plan(wc, 0, wc.space.n_configs, 200)
    assert p["tiles_per_wave"] == 1 and p["workgroups"] == 256 and p["n_units"] == 256
    assert p["dynamic_queue"] == 0 and p["live_chunk_list"] == 0
    # (the plan is that of a call with merge = 0: the running result is not one of the lists)
    # 256 lists of 256 keys: 8 workgroups merge 32 lists each, the last of them to finish merges
    # the eight results in the same launch; lists of 1024 keys (k = 1000): 16 workgroups merge 16
    # lists each and the last one the 16 results, which just fill its 128 KB
    assert p["merge_launches"] == 1
    assert plan(wl.large(), 0, 1 << 27, 1000)["merge_launches"] == 1
    assert plan(wl.streamed(), 0, 1 << 28, 4096)["merge_launches"] == 3      # 256 -> 64 -> 16 -> 4 -> 1
    # an empty range launches no sweep
    p = plan(wc, 77, 0, 200)
    assert p["workgroups"] == 0 and p["n_chunks"] == 0
    # errors of the calls it describes
    with pytest.raises(T.TunerError) as e:
        plan(wc, wc.space.n_configs - 5, 6, 200)
    assert e.value.code == T.TUNER_EINVAL
    with pytest.raises(T.TunerError) as e:
        plan(wc, 0, 10, T.TUNER_MAX_K + 1)
    assert e.value.code == T.TUNER_ETOOLARGE


def test_static_scratch_entry_point_argument_errors():
    L = T.load_library()
    w = wl.large()
    h = make_space(w.space)
    m = T.ModelHandle(4, w.model.widths, _FakeWeights())
    fake = C.c_void_p(0x2000)
    assert L.tuner_predict_topk_static(h.ptr, C.byref(m.c), 0, 256, 10, 0, None, fake, fake, None) == T.TUNER_EINVAL
    assert L.tuner_predict_topk_static(h.ptr, C.byref(m.c), 0, 256, 0, 0, fake, fake, fake, None) == T.TUNER_EINVAL
    assert L.tuner_predict_topk_static(h.ptr, C.byref(m.c), 0, 256, T.TUNER_MAX_K + 1, 0, fake, fake, fake, None) == T.TUNER_ETOOLARGE
    # k = 16384 needs 128 MiB of candidate pools: more than the static array
    assert T.tuner_workspace_bytes(h, m, 16384) > T.TUNER_STATIC_SCRATCH_BYTES
    assert L.tuner_predict_topk_static(h.ptr, C.byref(m.c), 0, 256, 16384, 0, fake, fake, fake, None) == T.TUNER_ETOOLARGE
    assert "static" in T.tuner_last_error() and str(T.TUNER_STATIC_SCRATCH_BYTES) in T.tuner_last_error()
    bad = T.ModelHandle(4, [13, 64, 64, 1], _FakeWeights())
    assert L.tuner_predict_topk_static(h.ptr, C.byref(bad.c), 0, 256, 10, 0, fake, fake, fake, None) == T.TUNER_EINVAL
    hdr = open(os.path.join(ROOT, "include", "tuner.h")).read()
    assert re.search(r"#define TUNER_STATIC_SCRATCH_BYTES \(64u << 20\)", hdr)
    assert T.TUNER_STATIC_SCRATCH_BYTES == 64 << 20


def test_prepare_and_prepared_calls_argument_errors():
    """tuner_prepare and the prepared entry points reject bad calls on the host like the calls
    they replace (no kernel is reached on a machine without a GPU)."""
    L = T.load_library()
    w = wl.paper_convolution()
    h = make_space(w.space)
    m = T.ModelHandle(11, w.model.widths, _FakeWeights())
    fake = C.c_void_p(0x4000)
    need = T.tuner_workspace_bytes(h, m, 200)
    assert L.tuner_prepare(None, C.byref(m.c), fake, need, None) == T.TUNER_EINVAL
    assert L.tuner_prepare(h.ptr, None, fake, need, None) == T.TUNER_EINVAL
    assert L.tuner_prepare(h.ptr, C.byref(m.c), None, need, None) == T.TUNER_EWORKSPACE
    assert L.tuner_prepare(h.ptr, C.byref(m.c), fake, 1024, None) == T.TUNER_EWORKSPACE
    assert L.tuner_prepare(h.ptr, C.byref(m.c), C.c_void_p(0x4010), need, None) == T.TUNER_EWORKSPACE
    bad = T.ModelHandle(11, [8, 30, 1], _FakeWeights())
    assert L.tuner_prepare(h.ptr, C.byref(bad.c), fake, need, None) == T.TUNER_EINVAL
    # header, tables and packed weights need far less than a top-k workspace
    assert T.tuner_workspace_bytes(h, m, 0) < need
    tk = L.tuner_predict_topk_prepared
    assert tk(h.ptr, C.byref(m.c), 0, 100, 200, 0, None, fake, fake, fake, need, None) == T.TUNER_EINVAL
    assert tk(h.ptr, C.byref(m.c), 0, 100, 0, 0, fake, fake, fake, fake, need, None) == T.TUNER_EINVAL
    assert tk(h.ptr, C.byref(m.c), 0, 100, T.TUNER_MAX_K + 1, 0, fake, fake, fake, fake, need, None) == T.TUNER_ETOOLARGE
    assert tk(h.ptr, C.byref(m.c), 131072 - 5, 6, 200, 0, fake, fake, fake, fake, need, None) == T.TUNER_EINVAL
    assert tk(h.ptr, C.byref(m.c), 0, 100, 200, 0, fake, fake, fake, fake, need - 1, None) == T.TUNER_EWORKSPACE
    pa = L.tuner_predict_all_prepared
    assert pa(h.ptr, C.byref(m.c), 0, 100, None, None, fake, need, None) == T.TUNER_EINVAL
    assert pa(h.ptr, C.byref(m.c), 0, 100, fake, None, None, need, None) == T.TUNER_EWORKSPACE
    assert pa(h.ptr, C.byref(m.c), 131072, 1, fake, None, fake, need, None) == T.TUNER_EINVAL


def test_profile_events_are_dropped_when_profiling_is_switched_off():
    T.tuner_profile_enable(True)
    assert T.tuner_profile_pending() == 0
    T.tuner_profile_enable(False)
    assert T.tuner_profile_pending() == 0


def test_which_parameters_are_constant_over_a_tile():
    """The fp32 matrix network takes the layer-1 share of the leading parameters whose stride
    is a multiple of 32 out of the matrix instructions when at most 8 parameters remain."""
    def hoisted(w, **kw):
        h = make_space(w.space)
        return T.tuner_hoisted_parameters(h, T.ModelHandle(w.model.n_members, w.model.widths, _FakeWeights(), **kw))
    assert hoisted(wl.large()) == 9            # 2^27: the last five parameters span 32 configurations
    assert hoisted(wl.streamed()) == 15        # 2^32: 20 parameters, the last five are boolean
    assert hoisted(wl.wide()) == 9
    assert hoisted(wl.conv_shaped()) == 4      # strides ..., 96, 48, 24, 12, 6, 3, 1
    assert hoisted(wl.tiny()) == 0             # 256 configurations: only one stride is a multiple of 32
    assert hoisted(wl.paper_stereo()) == 5     # strides 294912, 36864, 4608, 576, 288 | 144, 72, 36, 9, 3, 1
    assert hoisted(wl.large(), algo=T.TUNER_ALGO_SPLIT16) == 0
    assert hoisted(wl.large(), algo=T.TUNER_ALGO_VALU) == 0
    assert hoisted(wl.large(), precision=T.TUNER_BF16_MFMA) == 0


def test_which_parameters_come_from_the_table():
    """When the parameters that vary inside a tile span exactly 32 configurations, their layer-1
    share is tabulated per member, provided the larger members still fit LDS resident or as
    two stage buffers."""
    def tabulated(w, **kw):
        h = make_space(w.space)
        return T.tuner_tabulated_parameters(h, T.ModelHandle(w.model.n_members, w.model.widths, _FakeWeights(), **kw))
    assert tabulated(wl.large()) == 5              # 2^27: five boolean parameters = 32 configurations
    assert tabulated(wl.streamed()) == 5
    assert tabulated(wl.paper_convolution()) == 5
    assert tabulated(wl.wide()) == 0               # 128-wide members: the table would cost a stage buffer
    assert tabulated(wl.conv_shaped()) == 0        # low strides 12, 6, 3, 1: the pattern does not repeat
    assert tabulated(wl.paper_stereo()) == 0       # the low parameters span 288
    assert tabulated(wl.tiny()) == 0
    assert tabulated(wl.large(), algo=T.TUNER_ALGO_SPLIT16) == 0
    with pytest.raises(T.TunerError):
        tabulated(wl.large(), precision=7)


def test_tuner_stage_argument_errors_before_any_gpu_work():
    """Sampler, training, list evaluation, metric and second-stage entry points reject bad
    calls on the host (no HIP call is reached)."""
    L = T.load_library()
    w = wl.conv_shaped()
    h = make_space(w.space)
    fake = C.c_void_p(0x4000)
    # sampler
    assert T.tuner_sample_workspace_bytes(1000) % 256 == 0
    assert T.tuner_sample_workspace_bytes(1 << 24) >= 8 * (1 << 25)
    with pytest.raises(T.TunerError):
        T.tuner_sample_workspace_bytes(0)
    with pytest.raises(T.TunerError):
        T.tuner_sample_workspace_bytes((1 << 24) + 1)
    big = 1 << 40
    assert L.tuner_sample_valid(None, 1, 10, 100, fake, fake, fake, big, None) == T.TUNER_EINVAL
    assert L.tuner_sample_valid(h.ptr, 1, 10, 100, None, fake, fake, big, None) == T.TUNER_EINVAL
    assert L.tuner_sample_valid(h.ptr, 1, 0, 100, fake, fake, fake, big, None) == T.TUNER_EINVAL
    assert L.tuner_sample_valid(h.ptr, 1, 10, 9, fake, fake, fake, big, None) == T.TUNER_EINVAL
    assert L.tuner_sample_valid(h.ptr, 1, 10, (1 << 24) + 1, fake, fake, fake, big, None) == T.TUNER_ETOOLARGE
    assert L.tuner_sample_valid(h.ptr, 1, 10, 100, fake, fake, None, big, None) == T.TUNER_EWORKSPACE
    assert L.tuner_sample_valid(h.ptr, 1, 10, 100, fake, fake, fake, 64, None) == T.TUNER_EWORKSPACE
    assert L.tuner_sample_valid(h.ptr, 1, 10, 100, fake, fake, C.c_void_p(0x4010), big, None) == T.TUNER_EWORKSPACE
    # training
    need = T.tuner_train_workspace_bytes(h, 2000)
    assert need % 256 == 0 and need > 2000 * 4 * 16
    with pytest.raises(T.TunerError):
        T.tuner_train_workspace_bytes(h, (1 << 24) + 1)

    def train(space=h.ptr, E=11, H=30, n=2000, idx=fake, t=fake, parts=fake, w0=fake, opt=(10, 0.1, 0.5, 0, 0),
              out=fake, ws=fake, ws_bytes=need):
        o = T._TrainOptions(*opt) if opt is not None else None
        return L.tuner_train_ensemble(space, E, H, n, idx, t, parts, w0, C.byref(o) if o is not None else None,
                                      out, None, ws, ws_bytes, None)
    assert train(space=None) == T.TUNER_EINVAL
    assert train(w0=None) == T.TUNER_EINVAL
    assert train(out=None) == T.TUNER_EINVAL
    assert train(opt=None) == T.TUNER_EINVAL
    assert train(idx=None) == T.TUNER_EINVAL
    assert train(E=0) == T.TUNER_EINVAL
    assert train(H=0) == T.TUNER_EINVAL
    assert train(H=65) == T.TUNER_ETOOLARGE
    assert train(n=(1 << 24) + 1) == T.TUNER_ETOOLARGE
    assert train(opt=(-1, 0.1, 0.5, 0, 0)) == T.TUNER_EINVAL
    assert train(opt=(10, float("nan"), 0.5, 0, 0)) == T.TUNER_EINVAL
    assert train(opt=(10, 0.1, 0.5, 17, 0)) == T.TUNER_EINVAL
    assert train(opt=(10, 0.1, 0.5, 0, -1)) == T.TUNER_EINVAL
    assert train(ws=None) == T.TUNER_EWORKSPACE
    assert train(ws_bytes=need - 1) == T.TUNER_EWORKSPACE
    assert train(ws=C.c_void_p(0x4010)) == T.TUNER_EWORKSPACE
    assert "workspace" in T.tuner_last_error()
    # evaluation at a list, metric, second stage
    m = T.ModelHandle(8, w.model.widths, _FakeWeights())
    assert L.tuner_predict_indices(h.ptr, C.byref(m.c), 10, None, fake, None, fake, 1 << 30, None) == T.TUNER_EINVAL
    assert L.tuner_predict_indices(h.ptr, C.byref(m.c), 10, fake, None, None, fake, 1 << 30, None) == T.TUNER_EINVAL
    assert L.tuner_predict_indices(h.ptr, C.byref(m.c), 0, None, fake, None, None, 0, None) == T.TUNER_OK   # nothing to do
    assert L.tuner_predict_indices(h.ptr, C.byref(m.c), 10, fake, fake, None, fake, 16, None) == T.TUNER_EWORKSPACE
    assert L.tuner_mean_relative_error(10, None, fake, fake, fake, None) == T.TUNER_EINVAL
    assert L.tuner_mean_relative_error(10, fake, fake, None, fake, None) == T.TUNER_EINVAL
    assert L.tuner_mean_relative_error((1 << 31) + 1, fake, fake, fake, fake, None) == T.TUNER_ETOOLARGE
    assert L.tuner_best_of(10, None, fake, fake, None) == T.TUNER_EINVAL
    assert L.tuner_best_of(10, fake, None, fake, None) == T.TUNER_EINVAL
    assert L.tuner_best_of((1 << 31) + 1, fake, fake, fake, None) == T.TUNER_ETOOLARGE


def test_binding_fails_loudly_without_the_library(monkeypatch):
    monkeypatch.setattr(T, "_lib", None)
    monkeypatch.setattr(T, "LIB_PATH", "/nonexistent/libtuner_hip.so")
    with pytest.raises(ImportError):
        T.load_library()


def test_bench_refuses_more_than_one_gpu():
    """The benchmark is a one-GPU program: asking for more exits with a message, before any GPU call."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_header_is_plain_c_and_the_documented_call_sequence_links(tmp_path):
    """include/tuner.h compiles as C99 with warnings as errors, and a C program that makes the
    documented call sequence links against the library and runs its host-only part (space
    creation, size, workspace size, plan, error text) without a GPU."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "use_tuner.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "tuner.h"
int main(void) {
  const int32_t radices[3] = {4, 2, 8};
  const double values[14] = {1, 2, 4, 8, 0, 1, 1, 2, 3, 4, 5, 6, 7, 8};
  const int32_t scales[3] = {TUNER_SCALE_LOG2, TUNER_SCALE_LINEAR, TUNER_SCALE_LINEAR};
  const int32_t terms[14] = {0, 1, 2, 3, 0, 0, 0, 0, 0, 0, 0, 0, 1, 1};
  const int64_t bounds[1] = {3};
  tuner_space* space = NULL;
  if (tuner_space_create(3, radices, values, scales, 1, terms, bounds, &space) != TUNER_OK) return 1;
  uint64_t n = 0;
  if (tuner_space_size(space, &n) != TUNER_OK || n != 64) return 2;
  int32_t widths[3] = {3, 30, 1};
  float fake;                      /* never dereferenced on the host */
  tuner_model model = {11, 2, widths, &fake, TUNER_FP32, TUNER_ALGO_AUTO};
  size_t ws = tuner_workspace_bytes(space, &model, 10);
  if (ws == 0) return 3;
  tuner_sweep_plan_info info;
  if (tuner_sweep_plan(space, &model, 0, n, 10, &info) != TUNER_OK || info.workgroups < 1) return 4;
  /* a call that must fail on the host, before any GPU work: no workspace */
  int rc = tuner_predict_topk(space, &model, 0, n, 10, 0, &fake, (uint32_t*)&fake, (int32_t*)&fake, NULL, 0, NULL);
  if (rc != TUNER_EWORKSPACE || strlen(tuner_last_error()) == 0) return 5;
  printf("n=%llu ws=%zu workgroups=%d version=%s\n", (unsigned long long)n, ws, info.workgroups, tuner_version());
  tuner_space_destroy(space);
  return 0;
}
''')
    exe = tmp_path / "use_tuner"
    lib_dir = os.path.dirname(T.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                    str(src), "-o", str(exe), "-L", lib_dir, "-l:" + os.path.basename(T.LIB_PATH),
                    "-Wl,-rpath," + lib_dir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    assert out.startswith("n=64 ws=") and "workgroups=" in out
