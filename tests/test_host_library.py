"""CPU-side tests of libsconv: the library loads and exports the C ABI, its
lowering is bit-exact against the oracle's, the kernel packings round-trip, the
error paths answer with status codes, and the model matches the model oracle.
No kernel is launched here."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

from oracle import perf_model_oracle as pm
from paper_1608_01409_amd import binding as B
from paper_1608_01409_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def rand_w(layer, density, seed):
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((layer.K, layer.Cg, layer.R, layer.S)).astype(np.float32)
    if density < 1:
        w = np.where(rng.random(w.shape) < density, w, np.float32(0)).astype(np.float32)
    return w


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "sconv.h")).read()
    declared = set(re.findall(r"\b(sconv_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert B.strerror(0) == "ok" and "CSR" in B.strerror(B.ERR["CSR"])


CASES = [
    (wl.small_layer(), 0.4),
    (wl.small_layer(C=4, H=7, W=6, K=4, R=2, S=3, stride=2, pad=1, groups=2), 0.5),
    (wl.small_layer(C=2, H=13, W=12, K=2, R=5, S=4, stride=4, pad=0, groups=1), 0.7),
    (wl.small_layer(C=16, H=13, W=13, K=24, R=3, S=3, stride=1, pad=1, groups=2), 0.1),
    (wl.LAYERS["conv3"], 0.1),
    (wl.LAYERS["conv2"], 0.1),
    (wl.LAYERS["conv5"], 0.02),
    (wl.LAYERS["goog5x5"], 0.3),
    (wl.LAYERS["conv1"], 0.3),
]


@pytest.mark.parametrize("layer,density", CASES, ids=[f"{c[0].name}-{i}" for i, c in enumerate(CASES)])
def test_lowering_bit_exact_and_packings_round_trip(oracle, layer, density):
    w = rand_w(layer, density, seed=3)
    w[0, 0, 0, 0] = np.float32("nan")
    w[layer.K - 1, 0, 0, 0] = -0.0
    o_rowptr, o_col, o_val = oracle.csr_from_dense(layer, w)
    o_off = oracle.lower_offsets(layer, o_rowptr, o_col)
    h = B.sconv_create_csr(layer, w)
    rowptr, off, val = B.sconv_csr_export(h)
    assert np.array_equal(rowptr, o_rowptr)
    assert np.array_equal(off, o_off)
    assert np.array_equal(val.view(np.uint32), o_val.view(np.uint32))
    info = B.sconv_csr_info(h)
    assert info["nnz"] == len(o_val) and (info["OH"], info["OW"]) == (layer.OH, layer.OW)
    which = [2, 1]
    assert info["plan"]["kernel"] in (1, 3, 4)   # strided layers run the same kernels over their phase images
    for wh in which:
        r2, o2, v2 = B.sconv_csr_unpack(h, wh)
        assert np.array_equal(r2, o_rowptr) and np.array_equal(o2, o_off)
        assert np.array_equal(v2.view(np.uint32), o_val.view(np.uint32))
    # the same arrays through the CSR entry point
    h2 = B.sconv_create_csr_from_arrays(layer, o_rowptr, o_col, o_val)
    r3, o3, v3 = B.sconv_csr_export(h2)
    assert np.array_equal(r3, o_rowptr) and np.array_equal(o3, o_off)
    assert np.array_equal(v3.view(np.uint32), o_val.view(np.uint32))


PLANS = [
    dict(kernel=1, nt=4, cb=8, waves=8, cg=1, rows_w=6, t=3),
    dict(kernel=1, nt=4, cb=5, waves=4, cg=1, rows_w=4, t=3),
    dict(kernel=1, nt=8, cb=4, waves=8, cg=2, rows_w=6, t=3),
    dict(kernel=1, nt=8, cb=4, waves=8, cg=1, rows_w=3, t=6),
    dict(kernel=1, nt=1, cb=16, waves=8, cg=1, rows_w=8, t=3),
    dict(kernel=1, nt=2, cb=16, waves=4, cg=2, rows_w=8, t=3),
    dict(kernel=1, nt=4, cb=8, waves=8, cg=1, rows_w=4, t=2, band=7),   # two bands, the second ragged
    dict(kernel=1, nt=4, cb=16, waves=4, cg=1, rows_w=8, t=1, band=4),  # four bands
    dict(kernel=3, nt=4, cb=8, waves=8, cg=1, rows_w=6, t=3),           # flat streams
    dict(kernel=3, nt=4, cb=5, waves=4, cg=1, rows_w=4, t=3),
    dict(kernel=3, nt=4, cb=7, waves=8, cg=1, rows_w=8, t=2, band=7),
    dict(kernel=3, nt=4, cb=16, waves=16, cg=2, rows_w=16, t=1, band=7),
    dict(kernel=3, nt=4, cb=3, waves=4, cg=1, rows_w=8, t=3),
    dict(kernel=3, nt=4, cb=6, waves=8, cg=1, rows_w=4, t=3, band=7, strip=9),   # 3 strips of 9 columns for 13
    dict(kernel=3, nt=4, cb=6, waves=8, cg=2, rows_w=6, t=3, band=13, strip=9),  # two waves stacked: 14 rows
    dict(kernel=3, nt=4, cb=4, waves=4, cg=1, rows_w=2, t=7, band=8, strip=8),
    dict(kernel=3, nt=4, cb=3, waves=4, cg=1, rows_w=8, t=3, splits=3),          # channel blocks shared by 3 workgroups
]
PLANS += [dict(p, kernel=4) for p in PLANS if p["kernel"] == 3]                   # the flow variant packs the same way


@pytest.mark.parametrize("plan", PLANS, ids=[str(i) for i in range(len(PLANS))])
def test_explicit_plans_round_trip(oracle, plan):
    layer = wl.small_layer(C=32, H=13, W=13, K=50, R=3, S=3, stride=1, pad=1, groups=2)
    w = rand_w(layer, 0.15, seed=5)
    w[7] = 0  # an empty row
    o_rowptr, o_col, o_val = oracle.csr_from_dense(layer, w)
    o_off = oracle.lower_offsets(layer, o_rowptr, o_col)
    h = B.sconv_create_csr(layer, w, plan)
    got = B.sconv_csr_info(h)["plan"]
    assert got == {**dict(band=layer.OH, strip=0, splits=1), **plan}
    r, o, v = B.sconv_csr_unpack(h, 1)
    assert np.array_equal(r, o_rowptr) and np.array_equal(o, o_off)
    assert np.array_equal(v.view(np.uint32), o_val.view(np.uint32))


def test_explicit_zeros_survive_the_array_entry_point():
    layer = wl.small_layer(C=2, H=5, W=5, K=2, R=3, S=3, stride=1, pad=1, groups=1)
    rowptr = np.array([0, 2, 3], dtype=np.int32)
    colidx = np.array([0, 17, 4], dtype=np.int32)
    val = np.array([0.0, 1.5, -0.0], dtype=np.float32)
    h = B.sconv_create_csr_from_arrays(layer, rowptr, colidx, val)
    r, o, v = B.sconv_csr_export(h)
    assert np.array_equal(r, rowptr) and len(o) == 3
    assert np.array_equal(v.view(np.uint32), val.view(np.uint32))
    for wh in (1, 2):
        r2, o2, v2 = B.sconv_csr_unpack(h, wh)
        assert np.array_equal(o2, o) and np.array_equal(v2.view(np.uint32), val.view(np.uint32))


def test_error_paths():
    L = B.lib()
    layer = wl.small_layer()
    w = rand_w(layer, 0.5, seed=1)
    out = C.c_void_p()
    d = B.make_desc(layer)
    assert L.sconv_create_csr(None, w.ctypes.data_as(C.c_void_p), None, C.byref(out)) == B.ERR["NULL"]
    assert L.sconv_create_csr(C.byref(d), None, None, C.byref(out)) == B.ERR["NULL"]
    assert L.sconv_create_csr(C.byref(d), w.ctypes.data_as(C.c_void_p), None, None) == B.ERR["NULL"]
    for bad in (dict(C=0), dict(groups=3), dict(stride=0), dict(pad=-1), dict(R=20, pad=0), dict(K=5, groups=2)):
        with pytest.raises(B.SconvError) as e:
            B.sconv_create_csr(wl.small_layer(**bad), w)
        assert e.value.status == B.ERR["DESC"]
    # malformed CSR
    ncol = layer.Cg * layer.R * layer.S
    good_rp = np.array([0, 1, 1, 2, 2, 2, 3], dtype=np.int32)
    cases = [
        (np.array([1, 1, 1, 2, 2, 2, 3], dtype=np.int32), [0, 1, 2]),    # rowptr[0] != 0
        (np.array([0, 2, 1, 2, 2, 2, 3], dtype=np.int32), [0, 1, 2]),    # not monotone
        (good_rp, [0, ncol, 2]),                                         # column out of range
        (good_rp, [-1, 1, 2]),
        (np.array([0, 3, 3, 3, 3, 3, 3], dtype=np.int32), [0, 2, 2]),    # duplicate
        (np.array([0, 3, 3, 3, 3, 3, 3], dtype=np.int32), [0, 2, 1]),    # descending
    ]
    for rp, ci in cases:
        with pytest.raises(B.SconvError) as e:
            B.sconv_create_csr_from_arrays(layer, rp, np.array(ci, dtype=np.int32), np.ones(3, dtype=np.float32))
        assert e.value.status == B.ERR["CSR"], (rp, ci)
    # plans that cannot run
    with pytest.raises(B.SconvError) as e:
        B.sconv_create_csr(layer, w, dict(kernel=3, nt=8, cb=4, waves=8, cg=1, rows_w=6, t=3))  # flat streams: nt = 4 only
    assert e.value.status == B.ERR["PLAN"]
    # a strided layer runs the LDS kernels over its phase images, also on request
    hs = B.sconv_create_csr(wl.small_layer(stride=2), w, dict(kernel=1))
    assert B.sconv_csr_info(hs)["plan"]["kernel"] == 1
    with pytest.raises(B.SconvError) as e:
        B.sconv_create_csr(layer, w, dict(kernel=1, nt=4, cb=4, waves=8, cg=1, rows_w=6, t=1))  # too few chunks
    assert e.value.status == B.ERR["PLAN"]
    with pytest.raises(B.SconvError) as e:
        B.sconv_create_csr(layer, w, dict(kernel=1, nt=3, cb=4, waves=8, cg=1, rows_w=8, t=3))  # nt must divide 64
    assert e.value.status == B.ERR["PLAN"]
    # export capacity
    h = B.sconv_create_csr(layer, w)
    n = C.c_int64(1)
    rp = np.zeros(layer.K + 1, dtype=np.int32)
    one = np.zeros(1, dtype=np.int32)
    rc = L.sconv_csr_export(h.handle, rp.ctypes.data_as(C.c_void_p), one.ctypes.data_as(C.c_void_p),
                            one.ctypes.data_as(C.c_void_p), C.byref(n))
    assert rc == B.ERR["CAPACITY"] and n.value == B.sconv_csr_info(h)["nnz"]
    # forward argument checks happen before any device work
    assert L.sconv_forward(h.handle, None, None, 1, None) == B.ERR["NULL"]
    assert L.sconv_forward(h.handle, C.c_void_p(16), C.c_void_p(32), 0, None) == B.ERR["BATCH"]
    assert L.sconv_forward(None, C.c_void_p(16), C.c_void_p(32), 1, None) == B.ERR["NULL"]


def test_automatic_plans_for_the_benchmark_layers():
    for name in ("conv2", "conv3", "conv4", "conv5", "goog3x3", "goog5x5"):
        layer = wl.LAYERS[name]
        h = B.sconv_create_csr(layer, rand_w(layer, 0.1, seed=2))
        p = B.sconv_csr_info(h)["plan"]
        assert p["kernel"] in (1, 3, 4) and p["nt"] % 4 == 0, (name, p)
    h = B.sconv_create_csr(wl.LAYERS["conv1"], rand_w(wl.LAYERS["conv1"], 0.3, seed=2))
    assert B.sconv_csr_info(h)["plan"]["kernel"] in (3, 4)
    h = B.sconv_create_csr(wl.LAYERS["conv1"], rand_w(wl.LAYERS["conv1"], 0.3, seed=2), dict(kernel=2))
    assert B.sconv_csr_info(h)["plan"]["kernel"] == 2


# ------------------------------------------------------------------ model
def test_model_matches_oracle_with_paper_machine():
    layer = wl.LAYERS["conv5"]
    for (F, Bw, alpha) in [(2150e9, 122e9, 3.0), (62e9, 15e9, 1.2)]:
        m = B.sconv_machine(F, Bw, alpha, 2.0, 0, 0, 0, 0, 0)
        for N in (1, 144):
            for x in (0.001, 0.0197, 0.09, 0.3, 1.0):
                for lowered in (False, True):
                    for t_fixed in (0.0, 7e-6):
                        m.t_fixed = t_fixed
                        got = (B.sconv_model_predict_lowered if lowered else B.sconv_model_predict)(layer, N, x, machine=m)
                        ref = pm.predict(layer, N, x, F, Bw, alpha, 2.0, lowered=lowered, t_fixed=t_fixed)
                        for key, val in ref.items():
                            g = got[key]
                            if isinstance(val, bool):
                                assert bool(g) == val, key
                            elif math.isinf(val):
                                assert math.isinf(g)
                            else:
                                assert math.isclose(g, val, rel_tol=1e-12), (key, g, val, lowered, t_fixed)
                m.t_fixed = 0.0


def test_model_derived_alpha_and_realised_density():
    layer = wl.LAYERS["conv3"]
    m = B.sconv_machine_gfx950()
    assert m.alpha <= 0 and m.beta == 2.0
    a = pm.derive_alpha(m.dense_flops, m.fma_flops, m.lds_bytes_per_s, m.lds_bytes_per_fma, m.lane_efficiency)
    w = rand_w(layer, 0.1, seed=9)
    h = B.sconv_create_csr(layer, w)
    x = np.count_nonzero(w) / w.size
    got = B.sconv_model_predict(layer, 256, 0.5, csr=h)     # density argument replaced by the handle's
    ref = pm.predict(layer, 256, x, m.dense_flops, m.hbm_bytes_per_s, a, m.beta, t_fixed=m.t_fixed)
    assert m.t_fixed > 0
    assert math.isclose(got["density"], x, rel_tol=1e-12)
    for key in ("alpha", "t_dense", "t_sparse", "speedup", "x_upper", "x_lower", "actual_flops"):
        assert math.isclose(got[key], ref[key], rel_tol=1e-12), key
    L = B.lib()
    p = B.sconv_prediction()
    d = B.make_desc(layer)
    assert L.sconv_model_predict(C.byref(d), 0, 0.1, None, None, C.byref(p)) == B.ERR["BATCH"]
    assert L.sconv_model_predict(C.byref(d), 1, 0.1, None, None, None) == B.ERR["NULL"]


LOWER_CASES = [
    wl.small_layer(),
    wl.small_layer(C=4, H=7, W=6, K=4, R=2, S=3, stride=2, pad=1, groups=2),
    wl.small_layer(C=6, H=9, W=5, K=9, R=3, S=1, stride=3, pad=2, groups=3),
    wl.LAYERS["conv2"], wl.LAYERS["conv1"], wl.LAYERS["goog1x1"],
]


@pytest.mark.parametrize("layer", LOWER_CASES, ids=[f"{l.name}-{i}" for i, l in enumerate(LOWER_CASES)])
def test_lowering_alone_for_both_layouts_is_bit_exact(oracle, layer):
    """sconv_lower_offsets against the oracle's two lowerings, and its steps against the additivity they rest on."""
    w = rand_w(layer, 0.2, seed=13)
    rowptr, colidx, _ = oracle.csr_from_dense(layer, w)
    Wp = layer.W + 2 * layer.pad
    off, sy, sx = B.sconv_lower_offsets(layer, B.LAYOUT_CHW, rowptr, colidx)
    assert np.array_equal(off, oracle.lower_offsets(layer, rowptr, colidx))
    assert (sy, sx) == (layer.stride * Wp, layer.stride)
    off_h, sy, sx = B.sconv_lower_offsets(layer, B.LAYOUT_HWC, rowptr, colidx)
    assert np.array_equal(off_h, oracle.lower_offsets_hwc(layer, rowptr, colidx))
    assert (sy, sx) == (layer.stride * Wp * layer.C, layer.stride * layer.C)
    # the handle's own lowering is the CHW one
    h = B.sconv_create_csr(layer, w)
    assert np.array_equal(B.sconv_csr_export(h)[1], off)
    L = B.lib()
    d = B.make_desc(layer)
    buf = np.zeros(len(colidx) + 1, dtype=np.int32)
    args = (rowptr.ctypes.data_as(C.c_void_p), colidx.ctypes.data_as(C.c_void_p), buf.ctypes.data_as(C.c_void_p), None, None)
    assert L.sconv_lower_offsets(C.byref(d), 2, *args) == B.ERR["DESC"]            # no such layout
    assert L.sconv_lower_offsets(C.byref(d), 0, None, *args[1:]) == B.ERR["NULL"]
    bad = colidx.copy()
    bad[0] = layer.Cg * layer.R * layer.S
    assert L.sconv_lower_offsets(C.byref(d), 1, args[0], bad.ctypes.data_as(C.c_void_p), *args[2:]) == B.ERR["CSR"]


def test_gsl_decision_matches_oracle():
    cases = [(2150e9, 122e9, 3.0), (62e9, 15e9, 1.2)]
    for name in ("conv5", "conv2", "goog1x1_reduce", "goog1x1", "goog3x3"):
        layer = wl.LAYERS[name]
        for (F, Bw, alpha) in cases:
            m = B.sconv_machine(F, Bw, alpha, 2.0, 0, 0, 0, 0, 0)
            for N in (1, 64):
                for x in (0.004, 0.015, 0.05, 0.2, 0.34, 0.9, 1.0):
                    for st in (False, True):
                        act, pred = B.sconv_gsl_decide(layer, N, x, st, m)
                        assert act == pm.gsl_decide(layer, N, x, st, F, Bw, alpha), (name, F, N, x, st)
                        assert math.isclose(pred["x_lower"], 1 / alpha)
    # gfx950 defaults: the AlexNet layers have a useful range, the 1x1 reduce layer has none
    assert B.sconv_gsl_decide(wl.LAYERS["conv3"], 256, 0.1)[0] == "prune"
    assert B.sconv_gsl_decide(wl.LAYERS["goog1x1_reduce"], 64, 0.3)[0] == "exclude"
    L = B.lib()
    d = B.make_desc(wl.LAYERS["conv3"])
    a = C.c_int32()
    assert L.sconv_gsl_decide(C.byref(d), 1, 0.0, 0, None, C.byref(a), None) == B.ERR["DESC"]
    assert L.sconv_gsl_decide(C.byref(d), 1, 0.5, 0, None, None, None) == B.ERR["NULL"]


def test_balance_report_counts_streams_and_sees_skew():
    """sconv_csr_balance: chunk totals are consistent with the packing, per-block dealing keeps the waves of
    a workgroup level on a uniform mask, and a skewed mask (20 % empty rows, power-law row lengths) stays
    close to it: the rows are dealt so that each wave's stream is level block by block."""
    layer = wl.LAYERS["conv3"]
    plan = dict(kernel=3, nt=4, cb=22, waves=16, cg=1, rows_w=6, t=3)
    _, w = wl.make_case(1, 1, layer, 1, 0.10)
    h = B.sconv_create_csr(layer, w, plan)
    b = B.sconv_csr_balance(h)
    assert b["nnz"] == np.count_nonzero(w)
    assert b["nnz"] <= b["stream_entries"] < 1.03 * b["nnz"] and b["stream_entries"] % 4 == 0   # segments padded to fours
    n_wg, rg, nblk = 4, 16, 12   # 384 rows in tiles of 96; 256 channels in blocks of 22
    assert math.isclose(b["wave_mean"] * rg * 8, b["stream_entries"], rel_tol=1e-12)
    assert b["wave_mean"] <= b["simd_max"] <= b["wave_max"]
    assert b["wave_max"] / b["wave_mean"] < 1.10
    assert b["workgroup_mean"] <= b["workgroup_max"] < 1.05 * b["workgroup_mean"]
    assert math.isclose(b["workgroup_mean"] * n_wg, b["wave_max"], rel_tol=1e-12)
    _, ws = wl.make_case(3, 0, layer, 1, 0.10, skewed=True)
    hs = B.sconv_create_csr(layer, ws, plan)
    bs = B.sconv_csr_balance(hs)
    assert bs["nnz"] == np.count_nonzero(ws)
    assert bs["wave_max"] / bs["wave_mean"] < 1.25
    assert bs["workgroup_max"] / bs["workgroup_mean"] < 1.10
    # a handle without a kernel-3 packing has nothing to report
    hd = B.sconv_create_csr(layer, w, dict(kernel=2))
    out = B.sconv_balance()
    assert B.lib().sconv_csr_balance(hd.handle, C.byref(out)) == B.ERR["PLAN"]
    assert B.lib().sconv_csr_balance(h.handle, None) == B.ERR["NULL"]


def test_fc_planning_and_its_error_paths():
    """Host side of the fully connected path: which handles and batch sizes it takes, and that the tiling
    follows the batch (no GPU needed: planning and packing only)."""
    rng = np.random.default_rng(3)
    K, Cin = 300, 500
    w = np.where(rng.random((K, Cin, 1, 1)) < 0.1, rng.standard_normal((K, Cin, 1, 1)), 0).astype(np.float32)
    h = B.sconv_create_csr(B.fc_layer(Cin, K), w)
    p256 = B.sconv_fc_plan(h, 256)
    assert p256["kernel"] in (3, 4) and p256["nt"] == 4 and p256["t"] * p256["cg"] == 1 and p256["band"] == 1
    p1024 = B.sconv_fc_plan(h, 1024)
    assert p1024["t"] * p1024["cg"] == 4
    assert B.sconv_fc_plan(h, 2048)["t"] * B.sconv_fc_plan(h, 2048)["cg"] == 4   # two tiles of 1024
    # every packing unpacks to the canonical arrays, bit for bit
    er, eo, ev = B.sconv_csr_export(h)
    plans = {}
    for n in (2048, 256, 64, 8, 256, 2048, 12, 16, 20, 256, 8):   # earlier packings come back, the oldest are dropped
        p_n = B.sconv_fc_plan(h, n)
        assert plans.setdefault(n, p_n) == p_n
        r, o, v = B.sconv_csr_unpack(h, 3)
        assert np.array_equal(r, er) and np.array_equal(o, eo) and np.array_equal(v.view(np.uint32), ev.view(np.uint32)), n
    assert np.array_equal(eo, np.nonzero(w.reshape(K, Cin))[1])   # the lowered offset of a 1x1 layer on a 1x1 image is the feature
    L = B.lib()
    p = B.sconv_plan()
    for n in (0, 2, 6, 1028):   # not a multiple of 4; two tiles of 514 images, not a multiple of 4
        assert L.sconv_fc_plan(h.handle, n, C.byref(p)) == B.ERR["BATCH"], n
    assert L.sconv_fc_plan(h.handle, 256, None) == B.ERR["NULL"]
    conv = B.sconv_create_csr(wl.LAYERS["conv3"], np.zeros((384, 256, 3, 3), dtype=np.float32))
    assert L.sconv_fc_plan(conv.handle, 256, C.byref(p)) == B.ERR["DESC"]


def test_size_limits_are_refused_not_wrapped():
    """Maximum sizes: descriptions whose lowered offsets or CSR columns would leave int32 are refused with
    SCONV_ERR_RANGE; the largest ones below the limits are accepted (an empty pattern, so nothing is big)."""
    L = B.lib()

    def create_empty(**kw):
        layer = wl.small_layer("lim", **kw)
        d = B.make_desc(layer)
        rowptr = np.zeros(layer.K + 1, dtype=np.int32)
        out = C.c_void_p()
        rc = L.sconv_create_csr_from_arrays(C.byref(d), rowptr.ctypes.data_as(C.c_void_p), None, None, None, C.byref(out))
        if rc == B.SCONV_OK:
            L.sconv_destroy_csr(out)
        return rc

    # C * Hp * Wp must stay below 2^30
    assert create_empty(C=1024, H=1024, W=1024, K=1, R=1, S=1, stride=1, pad=0, groups=1) == B.ERR["RANGE"]
    assert create_empty(C=1023, H=1024, W=1024, K=1, R=1, S=1, stride=1, pad=0, groups=1) == B.SCONV_OK
    assert create_empty(C=1021, H=1024, W=1024, K=1, R=3, S=3, stride=1, pad=1, groups=1) == B.ERR["RANGE"]  # 1021 * 1026^2: the padding counts
    assert create_empty(C=1020, H=1024, W=1024, K=1, R=3, S=3, stride=1, pad=1, groups=1) == B.SCONV_OK
    # filter extents and padding are stored in 8 bits by the direct kernel's packing
    assert create_empty(C=1, H=300, W=300, K=1, R=256, S=1, stride=1, pad=0, groups=1) == B.ERR["RANGE"]
    assert create_empty(C=1, H=300, W=300, K=1, R=255, S=255, stride=1, pad=0, groups=1) == B.SCONV_OK
    assert create_empty(C=1, H=8, W=8, K=1, R=3, S=3, stride=1, pad=256, groups=1) == B.ERR["RANGE"]
    # K * Cg * R * S (the dense weight count) below 2^31
    assert create_empty(C=4096, H=16, W=16, K=65536, R=3, S=3, stride=1, pad=1, groups=1) == B.ERR["RANGE"]


@pytest.mark.parametrize("seed", range(12))
def test_random_layers_pack_and_unpack_bit_exactly(oracle, seed):
    """Seeded random layers (strides, pads, groups, odd sizes) and densities: the library's canonical arrays
    equal the oracle's, and whatever packing the library chooses unpacks to them again; the same for the
    fully connected packing at a few batch sizes."""
    rng = np.random.default_rng(9000 + seed)
    groups = int(rng.choice([1, 1, 2, 3]))
    R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    stride, pad = int(rng.choice([1, 1, 2, 3])), int(rng.integers(0, 3))
    H = max(int(rng.integers(1, 40)), R - 2 * pad, 1)
    W = max(int(rng.integers(1, 40)), S - 2 * pad, 1)
    layer = wl.small_layer("rnd", C=groups * int(rng.integers(1, 12)), H=H, W=W, K=groups * int(rng.integers(1, 30)),
                           R=R, S=S, stride=stride, pad=pad, groups=groups)
    dens = float(rng.choice([0.02, 0.1, 0.5, 1.0]))
    w = np.where(rng.random((layer.K, layer.Cg, R, S)) < dens, rng.standard_normal((layer.K, layer.Cg, R, S)), 0).astype(np.float32)
    o_rowptr, o_col, o_val = oracle.csr_from_dense(layer, w)
    o_off = oracle.lower_offsets(layer, o_rowptr, o_col)
    h = B.sconv_create_csr(layer, w)
    r, o, v = B.sconv_csr_export(h)
    assert np.array_equal(r, o_rowptr) and np.array_equal(o, o_off) and np.array_equal(v.view(np.uint32), o_val.view(np.uint32))
    for which in (1, 2):
        try:
            r2, o2, v2 = B.sconv_csr_unpack(h, which)
        except B.SconvError as e:   # a layer the LDS kernels cannot take has only the direct packing
            assert which == 1 and e.status == B.ERR["PLAN"]
            continue
        assert np.array_equal(r2, o_rowptr) and np.array_equal(o2, o_off), (which, layer)
        assert np.array_equal(v2.view(np.uint32), o_val.view(np.uint32))
    K, Cin = int(rng.integers(1, 70)), int(rng.integers(1, 90))
    wf = np.where(rng.random((K, Cin, 1, 1)) < dens, rng.standard_normal((K, Cin, 1, 1)), 0).astype(np.float32)
    hf = B.sconv_create_csr(B.fc_layer(Cin, K), wf)
    er, eo, ev = B.sconv_csr_export(hf)
    for n in (4, 64, 520, 2048):
        B.sconv_fc_plan(hf, n)
        r3, o3, v3 = B.sconv_csr_unpack(hf, 3)
        assert np.array_equal(r3, er) and np.array_equal(o3, eo) and np.array_equal(v3.view(np.uint32), ev.view(np.uint32)), n


def test_ranked_plans_start_with_the_cost_models_choice_and_all_pack():
    """sconv_rank_plans: distinct complete tilings, the first one the tiling an untuned handle uses for that
    batch size, every one accepted by sconv_create_csr and unpacking to the oracle's arrays."""
    from oracle import sconv_oracle as O
    layer = wl.small_layer("rank", C=24, H=13, W=13, K=40, R=3, S=3, stride=1, pad=1, groups=2)
    rng = np.random.default_rng(11)
    w = (rng.standard_normal((layer.K, layer.Cg, 3, 3)) * 0.01).astype(np.float32)
    w = np.where(rng.random(w.shape) < 0.2, w, 0).astype(np.float32)
    rp, ci, v = O.csr_from_dense(layer, w)
    off = O.lower_offsets(layer, rp, ci)
    h = B.sconv_create_csr(layer, w)
    for N in (1, 8, 256):
        plans = B.sconv_rank_plans(h, N, 12)
        assert 1 <= len(plans) <= 12
        assert len({tuple(sorted(p.items())) for p in plans}) == len(plans)
        for p in plans:
            assert p["kernel"] in (3, 4) and p["nt"] == 4 and all(p[k] > 0 for k in ("cb", "waves", "cg", "rows_w", "t", "band", "splits"))
            hp = B.sconv_create_csr(layer, w, p)
            assert B.sconv_csr_info(hp)["plan"] == p
            urp, uoff, uv = B.sconv_csr_unpack(hp, 1)
            assert np.array_equal(urp, rp) and np.array_equal(uoff, off) and np.array_equal(uv.view(np.uint32), v.view(np.uint32))
    # the first candidate for the batch size a new handle is planned for is the handle's own tiling
    assert B.sconv_rank_plans(h, 256, 4)[0] == B.sconv_csr_info(h)["plan"]
    assert len(B.sconv_rank_plans(h, 256, 0)) <= 8 and len(B.sconv_rank_plans(h, 256, 1000)) <= 32
    # handles without an LDS path have nothing to rank
    hd = B.sconv_create_csr(layer, w, dict(kernel=2))
    with pytest.raises(B.SconvError) as e:
        B.sconv_rank_plans(hd, 8)
    assert e.value.status == B.ERR["PLAN"]
