"""Pins for the performance-model oracle: the numbers Section 2.2 and
Section 3.2 print, read from tests/golden/paper_model_values.txt."""
import math
import os

import pytest

from oracle import perf_model_oracle as pm
from paper_1608_01409_amd import workloads as wl

GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "paper_model_values.txt")) as fh:
    for line in fh:
        line = line.split("#")[0].split()
        if len(line) == 2:
            GOLD[line[0]] = float(line[1])

CONV5 = wl.LAYERS["conv5"]


def test_conv5_counts_closed_form():
    flops, s_a, s_w = pm.layer_counts(CONV5, 1)
    assert flops == 2 * 256 * 192 * 9 * 169
    assert s_a == 4 * (384 * 169 + 256 * 169)
    assert s_w == 4 * 256 * 192 * 9


@pytest.mark.parametrize("plat", ["bdw", "atom"])
def test_upper_bound_of_useful_sparsity_matches_paper(plat):
    F, B = GOLD[f"{plat}_sgemm_gflops"] * 1e9, GOLD[f"{plat}_bw_gbs"] * 1e9
    p = pm.predict(CONV5, 1, 0.1, F, B, GOLD[f"{plat}_alpha"], GOLD["beta"])
    # the paper prints one significant digit
    assert round(p["x_upper"], 2) == GOLD[f"{plat}_conv5_x_upper"]
    # at x_upper the two sparse times are equal by definition
    q = pm.predict(CONV5, 1, p["x_upper"], F, B, GOLD[f"{plat}_alpha"], GOLD["beta"])
    assert math.isclose(q["t_sparse_compute"], q["t_sparse_bw"], rel_tol=1e-12)


def test_lower_bound_is_one_over_alpha():
    p = pm.predict(CONV5, 144, 0.1, GOLD["bdw_sgemm_gflops"] * 1e9, GOLD["bdw_bw_gbs"] * 1e9, GOLD["bdw_alpha"])
    assert round(p["x_lower"], 1) == GOLD["bdw_x_lower"]
    q = pm.predict(CONV5, 144, p["x_lower"], GOLD["bdw_sgemm_gflops"] * 1e9, GOLD["bdw_bw_gbs"] * 1e9, GOLD["bdw_alpha"])
    assert math.isclose(q["speedup"], 1.0, rel_tol=1e-12)


def test_projected_speedup_range_and_measured_point():
    F, B, a = GOLD["bdw_sgemm_gflops"] * 1e9, GOLD["bdw_bw_gbs"] * 1e9, GOLD["bdw_alpha"]
    lo = pm.predict(CONV5, 144, 0.15, F, B, a)["speedup"]
    hi = pm.predict(CONV5, 144, 0.05, F, B, a)["speedup"]
    assert round(lo) == GOLD["bdw_conv5_speedup_lo"] and round(hi) == GOLD["bdw_conv5_speedup_hi"]
    # measured 3.4x at x = 0.09 against the compute-bound projection 1/(alpha x)
    s = pm.predict(CONV5, 144, 0.09, F, B, a)["speedup"]
    assert math.isclose(s, 1 / (a * 0.09), rel_tol=1e-12)
    assert abs(s - GOLD["bdw_measured_speedup_x009"]) / GOLD["bdw_measured_speedup_x009"] < 0.15


def test_no_further_speedup_below_upper_bound_and_monotone_time():
    F, B, a = GOLD["bdw_sgemm_gflops"] * 1e9, GOLD["bdw_bw_gbs"] * 1e9, GOLD["bdw_alpha"]
    xs = [0.001, 0.005, 0.01, 0.02, 0.05, 0.1, 0.3, 0.5, 1.0]
    ps = [pm.predict(CONV5, 1, x, F, B, a) for x in xs]
    ts = [p["t_sparse"] for p in ps]
    assert all(t2 >= t1 for t1, t2 in zip(ts, ts[1:]))
    xu = ps[0]["x_upper"]
    below = [p for p, x in zip(ps, xs) if x < xu]
    assert all(p["bandwidth_bound"] for p in below)
    # speedup saturates: halving x below the bound gains < 5 %
    s1 = pm.predict(CONV5, 1, xu / 2, F, B, a)["speedup"]
    s2 = pm.predict(CONV5, 1, xu / 4, F, B, a)["speedup"]
    assert s2 / s1 < 1.05
    # effective = actual / density
    p = ps[5]
    assert math.isclose(p["effective_flops"] * 0.1, p["actual_flops"], rel_tol=1e-12)


def test_derived_alpha():
    a = pm.derive_alpha(F=100e12, fma_flops=80e12, lds_bytes_per_s=80e12, lds_bytes_per_fma=4.0, lane_efficiency=0.8)
    assert math.isclose(a, 100e12 / (0.8 * 40e12))
    a = pm.derive_alpha(F=100e12, fma_flops=30e12, lds_bytes_per_s=80e12, lds_bytes_per_fma=4.0, lane_efficiency=1.0)
    assert math.isclose(a, 100 / 30)


def test_gsl_rules_on_the_papers_examples():
    """Section 2.3: the 1x1 reduce layer that is bandwidth bound before pruning is excluded; conv5 is pruned
    inside its useful range, stopped below x_upper (~0.02 on the Xeon) and given up above 1/alpha = 0.3."""
    F, B, a = GOLD["bdw_sgemm_gflops"] * 1e9, GOLD["bdw_bw_gbs"] * 1e9, GOLD["bdw_alpha"]
    reduce_ = wl.LAYERS["goog1x1_reduce"]
    dense = pm.predict(reduce_, 1, 1.0, F, B, 1.0)
    assert dense["t_dense"] < dense["t_sparse_bw"]            # bandwidth bound even when dense
    assert (pm.gsl_decide(reduce_, 1, 0.3, False, F, B, a) != "exclude") == bool(GOLD["inception_4a_5x5_reduce_has_potential"])
    assert (pm.gsl_decide(CONV5, 1, 0.3, False, F, B, a) != "exclude") == bool(GOLD["alexnet_conv5_has_potential"])
    assert pm.gsl_decide(CONV5, 1, 0.10, False, F, B, a) == "prune"
    assert pm.gsl_decide(CONV5, 1, 0.10, True, F, B, a) == "prune"       # stabilised inside the range: keep it sparse
    assert pm.gsl_decide(CONV5, 1, 0.015, False, F, B, a) == "stop"      # below x_upper ~ 0.02
    assert pm.gsl_decide(CONV5, 1, 0.5, False, F, B, a) == "prune"       # still moving
    assert pm.gsl_decide(CONV5, 1, 0.5, True, F, B, a) == "restore_dense"  # stuck above 1/alpha ~ 0.33
    # the decision is monotone in the density once stabilised: stop, prune, restore
    order = {"stop": 0, "prune": 1, "restore_dense": 2}
    seq = [order[pm.gsl_decide(CONV5, 1, x, True, F, B, a)] for x in (0.005, 0.01, 0.03, 0.1, 0.3, 0.34, 0.6, 1.0)]
    assert seq == sorted(seq) and seq[0] == 0 and seq[-1] == 2


# ------------------------------------------------------------ the "lowered" curve of the Section 2.2 figure
def test_lowered_counts_closed_form():
    """Lowering turns the C x H x W input into a (C*R*S) x (OH*OW) matrix: for conv5 (3x3, stride 1, pad 1)
    every input element appears 9 times."""
    flops, s_a, s_w = pm.layer_counts(CONV5, 1, lowered=True)
    d_flops, d_s_a, d_s_w = pm.layer_counts(CONV5, 1)
    assert (flops, s_w) == (d_flops, d_s_w)                 # the arithmetic and the weights do not change
    assert s_a == 4 * (384 * 9 * 169 + 256 * 169)
    conv1 = wl.LAYERS["conv1"]                              # strided: 121 taps, 55 x 55 windows
    assert pm.layer_counts(conv1, 2, lowered=True)[1] == 4 * 2 * (3 * 121 * 55 * 55 + 96 * 55 * 55)


@pytest.mark.parametrize("plat", ["bdw", "atom"])
def test_lowered_curve_saturates_at_a_higher_density_than_direct(plat):
    """What the figure shows for conv5: both curves coincide while compute bound; the lowered one turns
    bandwidth bound at a higher density and its plateau is lower by the ratio of the activation bytes."""
    F, B, a = GOLD[f"{plat}_sgemm_gflops"] * 1e9, GOLD[f"{plat}_bw_gbs"] * 1e9, GOLD[f"{plat}_alpha"]
    direct = pm.predict(CONV5, 1, 0.2, F, B, a)
    lowered = pm.predict(CONV5, 1, 0.2, F, B, a, lowered=True)
    assert lowered["x_upper"] > 3 * direct["x_upper"]
    assert lowered["x_lower"] == direct["x_lower"]
    x_hi = 1.5 * lowered["x_upper"]                         # both compute bound
    assert pm.predict(CONV5, 1, x_hi, F, B, a, lowered=True)["speedup"] == pm.predict(CONV5, 1, x_hi, F, B, a)["speedup"]
    x_lo = 0.5 * direct["x_upper"]                          # both bandwidth bound
    pd, pl = pm.predict(CONV5, 1, x_lo, F, B, a), pm.predict(CONV5, 1, x_lo, F, B, a, lowered=True)
    assert pd["bandwidth_bound"] and pl["bandwidth_bound"] and pl["speedup"] < pd["speedup"]
    beta = 2.0
    want = (pd["bytes_act"] + beta * x_lo * pd["bytes_w"]) / (pl["bytes_act"] + beta * x_lo * pl["bytes_w"])
    assert math.isclose(pl["speedup"] / pd["speedup"], want, rel_tol=1e-12)
    # direct convolution keeps its advantage over the whole "typical" range only where lowering is bandwidth bound
    for x in (0.05, 0.1, 0.15):
        assert pm.predict(CONV5, 1, x, F, B, a, lowered=True)["speedup"] <= pm.predict(CONV5, 1, x, F, B, a)["speedup"]


def test_fixed_time_only_shifts_the_sparse_time():
    F, B, a = GOLD["bdw_sgemm_gflops"] * 1e9, GOLD["bdw_bw_gbs"] * 1e9, GOLD["bdw_alpha"]
    p0 = pm.predict(CONV5, 8, 0.1, F, B, a)
    p1 = pm.predict(CONV5, 8, 0.1, F, B, a, t_fixed=5e-6)
    assert p1["t_sparse"] == p0["t_sparse"] + 5e-6 and p1["t_dense"] == p0["t_dense"]
    assert p1["x_upper"] == p0["x_upper"] and p1["x_lower"] == p0["x_lower"]
    assert math.isclose(p1["speedup"], p0["t_dense"] / (p0["t_sparse"] + 5e-6), rel_tol=1e-15)
