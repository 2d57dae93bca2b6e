#!/usr/bin/env python3
"""Measurement reports beyond the one-line benchmark: the density sweep with the
roofline model's prediction and the dense-convolution crossover (Section 2.2,
Section 3.2 / Figure 5 of the paper), the skewed guided-pruning-like patterns,
and the GoogLeNet-like and strided layers.

    python -m paper_1608_01409_amd.report latency|sweep|skewed|extra|onebyone|fc|tune|all [--iters K]

Every input is seeded and synthetic (paper_1608_01409_amd/workloads.py).  The
dense reference is the vendor's fp32 convolution reached through
torch.nn.functional.conv2d (the paper uses the vendor SGEMM as its proxy for
dense convolution, Section 3.2).  Prints a text table and one JSON line per
table row.
"""
from __future__ import annotations

import argparse
import json
import math
import sys

import numpy as np
import torch

from . import binding as B
from . import workloads as wl


def time_gpu(fn, iters: int, warm: int = 3, warm_ms: float = 30.0) -> float:
    """Mean milliseconds per call, HIP events on the current stream, back-to-back launches.  The warm-up
    runs for at least warm_ms of GPU time: after the host-side packing of a new handle the GPU has dropped
    to a low clock state and the first milliseconds of work run well below the sustained rate."""
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    fn()                       # a first call may pack and upload: keep that out of the estimate below
    torch.cuda.synchronize()
    e0.record()
    for _ in range(warm):
        fn()
    e1.record()
    torch.cuda.synchronize()
    per_call = max(e0.elapsed_time(e1) / warm, 1e-3)
    for _ in range(int(warm_ms / per_call) + 1):   # no synchronisation between the warm-up and the timed calls
        fn()
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def time_sparse(layer, w, xd, iters, plan=None, tune=0):
    """tune > 0: the library times that many of its best-ranked tilings first and keeps the fastest (sconv_tune)."""
    h = B.sconv_create_csr(layer, w, plan)
    info = B.sconv_csr_info(h)
    out = torch.empty((xd.shape[0], layer.K, info["OH"], info["OW"]), dtype=torch.float32, device="cuda")
    if tune > 0 and plan is None:
        B.sconv_tune(h, xd, out, max_plans=tune)
    ms = time_gpu(lambda: B.sconv_forward(h, xd, out), iters)
    return ms, B.sconv_csr_info(h), h   # the tiling is settled by the first forward call


def time_dense(layer, xd, iters):
    """Vendor fp32 dense convolution of the same shape (all weights nonzero)."""
    torch.backends.cudnn.allow_tf32 = False
    torch.backends.cuda.matmul.allow_tf32 = False
    wd = torch.randn((layer.K, layer.Cg, layer.R, layer.S), device="cuda") * 0.01
    fn = lambda: torch.nn.functional.conv2d(xd, wd, None, layer.stride, layer.pad, 1, layer.groups)
    return time_gpu(fn, iters, warm=5)


def time_dense_gemm(layer, N, iters):
    """The paper's proxy for dense convolution (Section 3.2): the vendor's fp32 matrix product of the lowered
    shapes, per group [Kg x Cg*R*S] x [Cg*R*S x OH*OW*N]; the lowering itself is not timed."""
    torch.backends.cuda.matmul.allow_tf32 = False
    kdim, cols = layer.Cg * layer.R * layer.S, layer.OH * layer.OW * N
    a = torch.randn((layer.Kg, kdim), device="cuda") * 0.01
    b = torch.randn((kdim, cols), device="cuda")
    c = torch.empty((layer.Kg, cols), device="cuda")
    return layer.groups * time_gpu(lambda: torch.matmul(a, b, out=c), iters, warm=5)


def crossover(xs, t_sparse, t_dense):
    """Density at which the sparse time reaches the dense time: log-linear interpolation between the two
    sweep points that bracket it; None if sparse stays faster (or slower) over the whole sweep."""
    for i in range(len(xs) - 1):
        a, b = t_sparse[i] - t_dense, t_sparse[i + 1] - t_dense
        if a <= 0 < b:
            la, lb = math.log(xs[i]), math.log(xs[i + 1])
            ta, tb = math.log(t_sparse[i]), math.log(t_sparse[i + 1])
            f = (math.log(t_dense) - ta) / (tb - ta)
            return math.exp(la + f * (lb - la))
    return None


def knee(xs, ts):
    """Density below which the measured time stops falling: where the line through the compute-bound points
    (x >= 0.1, least squares of t against x) meets the floor (the time at the lowest density)."""
    pts = [(x, t) for x, t in zip(xs, ts) if 0.09 <= x <= 0.55]
    if len(pts) < 2:
        return None, None, None
    mx, mt = sum(p[0] for p in pts) / len(pts), sum(p[1] for p in pts) / len(pts)
    slope = sum((p[0] - mx) * (p[1] - mt) for p in pts) / sum((p[0] - mx) ** 2 for p in pts)
    icpt = mt - slope * mx
    floor = ts[0]
    return (floor - icpt) / slope if slope > 0 else None, icpt, slope


def emit(row):
    print(json.dumps(row), flush=True)


def report_sweep(iters, tune=16):
    print(f"# density sweep, AlexNet conv2-5, batch 256 (configuration 3); tilings: the fastest of the library's {tune} "
          "best-ranked per point (sconv_tune); t_model = Section 2.2's max(compute, bandwidth) + the machine's t_fixed")
    print(f"{'layer':6s} {'x':>5s} {'nnz':>8s} {'t_meas us':>10s} {'t_model us':>10s} {'meas/model':>10s} {'TFLOP/s':>8s} "
          f"{'t_dense us':>10s} {'speedup':>8s} {'model spd':>9s}")
    for li, (name, N, _) in enumerate(wl.CONFIGS[1]):
        layer = wl.LAYERS[name]
        xs, ts = [], []
        x0, _ = wl.make_case(2, li, layer, N, 0.1)
        xd = torch.from_numpy(x0).cuda()
        t_conv, t_gemm = time_dense(layer, xd, iters) * 1e-3, time_dense_gemm(layer, N, iters) * 1e-3
        t_dense = min(t_conv, t_gemm)   # the faster of the vendor's convolution and its matrix product of the lowered shapes
        print(f"{name}: dense fp32 convolution {t_conv*1e6:.1f} us, matrix product of the lowered shapes {t_gemm*1e6:.1f} us")
        pred1 = None
        for dens in wl.SWEEP_DENSITIES:
            _, w = wl.make_case(2, li, layer, 1, dens)
            ms, info, h = time_sparse(layer, w, xd, iters, tune=tune)
            pred = B.sconv_model_predict(layer, N, dens, h)
            pred1 = pred
            flops = 2.0 * info["nnz"] * info["OH"] * info["OW"] * N
            xs.append(pred["density"])
            ts.append(ms * 1e-3)
            row = dict(report="sweep", layer=name, density=dens, realised=pred["density"], nnz=info["nnz"],
                       t_meas_us=ms * 1e3, t_model_us=pred["t_sparse"] * 1e6, tflops=flops / ms / 1e9,
                       t_dense_us=t_dense * 1e6, speedup=t_dense / (ms * 1e-3), model_speedup=pred["speedup"],
                       bandwidth_bound=bool(pred["bandwidth_bound"]), plan=info["plan"])
            print(f"{name:6s} {dens:5.2f} {info['nnz']:8d} {ms*1e3:10.1f} {pred['t_sparse']*1e6:10.1f} {ms*1e-3/pred['t_sparse']:10.2f} "
                  f"{flops/ms/1e9:8.2f} {t_dense*1e6:10.1f} {t_dense/(ms*1e-3):8.2f} {pred['speedup']:9.2f}")
            emit(row)
        xc = crossover(xs, ts, t_dense)
        # model's crossover with the measured dense rate in place of the default
        m = B.sconv_machine_gfx950()
        flops_dense = pred1["flops_dense"]
        m.dense_flops = flops_dense / t_dense
        pm = B.sconv_model_predict(layer, N, 0.1, None, m)
        ratio = (xc / pm["x_lower"]) if xc else None
        # alpha as the paper measures it (Section 3.2): dense rate over the sparse kernel's rate at x = 1
        alpha_meas = (flops_dense / t_dense) / (flops_dense / ts[-1])
        xk, icpt, slope = knee(xs, [t * 1e6 for t in ts])
        pl = B.sconv_model_predict_lowered(layer, N, 0.1, None, m)
        print(f"{name}: measured crossover x = {xc}, model x_lower = {pm['x_lower']:.3f} (alpha {pm['alpha']:.2f} from the "
              f"ceilings with lane_efficiency CALIBRATED to the x = 1 plateau, as the paper takes alpha from its measured plateau; "
              f"{alpha_meas:.2f} from this run's plateau; dense {m.dense_flops/1e12:.1f} TFLOP/s measured), ratio {ratio}")
        print(f"{name}: upper bound of useful sparsity: model x_upper = {pm['x_upper']:.4f}; measured knee x = {xk if xk is None else round(xk, 4)} "
              f"(floor {ts[0]*1e6:.1f} us at x = {xs[0]:.3f}; compute-bound line {icpt:.1f} us + {slope:.0f} us * x), "
              f"ratio {None if not xk else round(xk / pm['x_upper'], 2)}; density at which the line's compute part alone equals the floor "
              f"(the section's own definition: compute time = bandwidth time) {ts[0]*1e6/slope:.4f}, ratio {ts[0]*1e6/slope/pm['x_upper']:.2f}; "
              f"on lowered tensors the model's x_upper would be {pl['x_upper']:.4f}")
        emit(dict(report="crossover", layer=name, measured=xc, model_x_lower=pm["x_lower"], model_x_upper=pm["x_upper"],
                  measured_knee=xk, fixed_us=icpt, us_per_unit_density=slope, lowered_x_upper=pl["x_upper"],
                  alpha=pm["alpha"], alpha_from_plateau=alpha_meas, dense_tflops=m.dense_flops / 1e12, ratio=ratio,
                  t_dense_conv_us=t_conv * 1e6, t_dense_gemm_us=t_gemm * 1e6))


def report_latency():
    """Configuration 1: one image through conv3, the latency case.  Median of 200 single launches, each
    bracketed by its own pair of events, after 20 warm-up launches."""
    print("# latency: conv3, batch 1, density 0.10 (configuration 1)")
    name, N, dens = wl.CONFIGS[0][0]
    layer = wl.LAYERS[name]
    x, w = wl.make_case(0, 0, layer, N, dens)
    xd = torch.from_numpy(x).cuda()
    h = B.sconv_create_csr(layer, w)
    out = B.sconv_forward(h, xd)
    for _ in range(20):
        B.sconv_forward(h, xd, out)
    torch.cuda.synchronize()
    ts = []
    for _ in range(200):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B.sconv_forward(h, xd, out)
        e1.record()
        e1.synchronize()
        ts.append(e0.elapsed_time(e1))
    med = float(np.median(ts))
    info = B.sconv_csr_info(h)
    flops = 2.0 * info["nnz"] * info["OH"] * info["OW"] * N
    # the same launches back to back between one pair of events: what a stream of requests sees, without the
    # 6-10 us that an event pair around a single launch adds (the wait for an idle queue to pick the launch up)
    b2b = time_gpu(lambda: B.sconv_forward(h, xd, out), 200)
    B.sconv_tune(h, xd, out, 24)
    tuned = time_gpu(lambda: B.sconv_forward(h, xd, out), 200)
    print(f"{name}: N {N} nnz {info['nnz']}: one launch between two events, median of 200: {med*1e3:.1f} us (min {min(ts)*1e3:.1f}), "
          f"{flops/med/1e6:.1f} GFLOP/s; 200 launches back to back: {b2b*1e3:.1f} us each; the same with the tiling tuned "
          f"(sconv_tune, 24 candidates): {tuned*1e3:.1f} us; plan {info['plan']} -> {B.sconv_csr_info(h)['plan']}")
    emit(dict(report="latency", layer=name, N=N, nnz=info["nnz"], median_us=med * 1e3, min_us=min(ts) * 1e3,
              back_to_back_us=b2b * 1e3, tuned_back_to_back_us=tuned * 1e3, gflops=flops / med / 1e6, plan=info["plan"]))


def report_skewed(iters):
    print("# skewed per-row densities, 20% empty rows, batch 256 (configuration 4); nonzeros clustered into active input "
          "channels, or into one run of kernel positions per active channel")
    for li, name, cluster in ((0, "conv3", "channels"), (1, "conv4", "channels"), (0, "conv3", "positions"), (1, "conv4", "positions")):
        layer = wl.LAYERS[name]
        x, w = wl.make_case(3, li, layer, 256, 0.10, skewed=True, cluster=cluster)
        xd = torch.from_numpy(x).cuda()
        nnz_row = (w.reshape(layer.K, -1) != 0).sum(1)
        ms, info, _ = time_sparse(layer, w, xd, iters)
        flops = 2.0 * info["nnz"] * info["OH"] * info["OW"] * 256
        # the same number of nonzeros spread uniformly, for comparison
        dens = info["nnz"] / w.size
        _, wu = wl.make_case(3, li + 2, layer, 1, dens)
        msu, infou, _ = time_sparse(layer, wu, xd, iters)
        flu = 2.0 * infou["nnz"] * infou["OH"] * infou["OW"] * 256
        row = dict(report="skewed", layer=name, cluster=cluster, nnz=info["nnz"], empty_rows=int((nnz_row == 0).sum()),
                   max_row=int(nnz_row.max()), mean_row=float(nnz_row.mean()), t_us=ms * 1e3, tflops=flops / ms / 1e9,
                   uniform_t_us=msu * 1e3, uniform_tflops=flu / msu / 1e9, plan=info["plan"])
        print(f"{name} ({cluster}): nnz {info['nnz']} rows empty {row['empty_rows']} max/mean {row['max_row']}/{row['mean_row']:.0f}: "
              f"{ms*1e3:.1f} us {row['tflops']:.2f} TFLOP/s; uniform mask of the same density: {msu*1e3:.1f} us "
              f"{row['uniform_tflops']:.2f} TFLOP/s")
        emit(row)


def report_extra(iters, cfg=4, title="# GoogLeNet-inception-like and strided layers, batch 64 (configuration 5)"):
    print(title)
    for li, (name, N, dens) in enumerate(wl.CONFIGS[cfg]):
        layer = wl.LAYERS[name]
        x, w = wl.make_case(cfg, li, layer, N, dens)
        xd = torch.from_numpy(x).cuda()
        ms, info, h = time_sparse(layer, w, xd, iters)
        t_conv, t_gemm = time_dense(layer, xd, iters), time_dense_gemm(layer, N, iters)
        t_dense = min(t_conv, t_gemm)
        flops = 2.0 * info["nnz"] * info["OH"] * info["OW"] * N
        pred = B.sconv_model_predict(layer, N, dens, h)
        hbm = pred["bytes_act"] / (ms * 1e-3) / 1e12
        row = dict(report="extra", layer=name, N=N, density=dens, nnz=info["nnz"], t_us=ms * 1e3, tflops=flops / ms / 1e9,
                   t_dense_us=t_dense * 1e3, t_dense_conv_us=t_conv * 1e3, t_dense_gemm_us=t_gemm * 1e3,
                   speedup=t_dense / ms, t_model_us=pred["t_sparse"] * 1e6,
                   model_bandwidth_bound=bool(pred["bandwidth_bound"]), model_x_upper=pred["x_upper"],
                   model_x_lower=pred["x_lower"], activation_tb_per_s=hbm, plan=info["plan"])
        print(f"{name}: N {N} x {dens} nnz {info['nnz']}: {ms*1e3:.1f} us {row['tflops']:.2f} TFLOP/s "
              f"({hbm:.2f} TB/s of activations), dense {t_dense*1e3:.1f} us (convolution {t_conv*1e3:.1f}, matrix product {t_gemm*1e3:.1f}), speedup {t_dense/ms:.2f}, model {pred['t_sparse']*1e6:.1f} us "
              f"({'bandwidth' if pred['bandwidth_bound'] else 'compute'} bound, useful x in ({pred['x_upper']:.3f}, {pred['x_lower']:.3f})), "
              f"plan {info['plan']}")
        emit(row)


def report_fc(iters):
    print("# fully connected layers of AlexNet as sparse x dense products (feature-major activations)")
    for i, (name, N, dens) in enumerate(wl.FC_CONFIG):
        C_in, K = wl.FC_LAYERS[name]
        x_t, w = wl.make_fc_case(i, name, N, dens)
        xd = torch.from_numpy(x_t).cuda()
        h = B.sconv_create_csr(B.fc_layer(C_in, K), w.reshape(K, C_in, 1, 1), dict(kernel=2))
        out = torch.empty((K, N), dtype=torch.float32, device="cuda")
        ms = time_gpu(lambda: B.sconv_fc_forward(h, xd, None, False, out), iters)
        wd = torch.from_numpy(w).cuda()
        torch.backends.cuda.matmul.allow_tf32 = False
        ms_dense = time_gpu(lambda: torch.matmul(wd, xd), iters, warm=5)
        nnz = int(np.count_nonzero(w))
        flops = 2.0 * nnz * N
        plan = B.sconv_fc_plan(h, N)
        # Section 2.2's model on the layer as a 1x1 convolution of 1x1 images, with the measured dense rate
        m = B.sconv_machine_gfx950()
        m.dense_flops = 2.0 * K * C_in * N / (ms_dense * 1e-3)
        pred = B.sconv_model_predict(B.fc_layer(C_in, K), N, nnz / w.size, None, m)
        row = dict(report="fc", layer=name, N=N, density=dens, nnz=nnz, t_us=ms * 1e3, tflops=flops / ms / 1e9,
                   t_dense_us=ms_dense * 1e3, dense_tflops=2.0 * K * C_in * N / ms_dense / 1e9, speedup=ms_dense / ms,
                   weight_gb_per_s=8.0 * nnz / (ms * 1e-3) / 1e9, t_model_us=pred["t_sparse"] * 1e6,
                   model_bandwidth_bound=bool(pred["bandwidth_bound"]), model_x_upper=pred["x_upper"],
                   model_x_lower=pred["x_lower"], plan=plan)
        print(f"{name}: N {N} x {dens} nnz {nnz}: {ms*1e3:.1f} us {row['tflops']:.2f} TFLOP/s, dense fp32 matmul {ms_dense*1e3:.1f} us "
              f"({row['dense_tflops']:.1f} TFLOP/s), speedup {ms_dense/ms:.2f}, model {pred['t_sparse']*1e6:.1f} us "
              f"({'bandwidth' if pred['bandwidth_bound'] else 'compute'} bound, useful x in ({pred['x_upper']:.3f}, {pred['x_lower']:.3f})), plan {plan}")
        emit(row)


TUNE_CASES = [("conv2", 256, 0.1), ("conv3", 256, 0.1), ("conv4", 256, 0.1), ("conv5", 256, 0.1), ("conv3", 64, 0.1),
              ("conv3", 16, 0.1), ("conv3", 1, 0.1), ("conv5", 64, 0.1), ("conv2", 64, 0.1), ("goog3x3", 64, 0.2),
              ("goog5x5", 64, 0.3), ("conv1", 64, 0.3)]


def report_tune(iters, max_plans=24):
    """The cost model's tiling against the measured choice (sconv_tune / sconv_fc_tune) on one box."""
    print(f"# tiling chosen by the cost model against the fastest of its {max_plans} best-ranked tilings, timed (sconv_tune)")
    for i, (name, N, dens) in enumerate(TUNE_CASES):
        layer = wl.LAYERS[name]
        x, w = wl.make_case(1, i, layer, N, dens)
        xd = torch.from_numpy(x).cuda()
        h = B.sconv_create_csr(layer, w)
        out = B.sconv_forward(h, xd)
        ms0 = time_gpu(lambda: B.sconv_forward(h, xd, out), iters)
        p0 = B.sconv_csr_info(h)["plan"]
        B.sconv_tune(h, xd, out, max_plans)
        ms1 = time_gpu(lambda: B.sconv_forward(h, xd, out), iters)
        p1 = B.sconv_csr_info(h)["plan"]
        print(f"{name} N {N}: model's choice {ms0*1e3:.1f} us, tuned {ms1*1e3:.1f} us ({100*(ms1/ms0-1):+.1f} %)"
              f"{'' if p0 == p1 else f', {p0} -> {p1}'}")
        emit(dict(report="tune", layer=name, N=N, density=dens, t_model_choice_us=ms0 * 1e3, t_tuned_us=ms1 * 1e3,
                  plan_model=p0, plan_tuned=p1))
    for i, (name, N, dens) in enumerate(wl.FC_CONFIG):
        C_in, K = wl.FC_LAYERS[name]
        x_t, w = wl.make_fc_case(i, name, N, dens)
        xd = torch.from_numpy(x_t).cuda()
        h = B.sconv_create_csr(B.fc_layer(C_in, K), w.reshape(K, C_in, 1, 1), dict(kernel=2))
        out = B.sconv_fc_forward(h, xd)
        ms0 = time_gpu(lambda: B.sconv_fc_forward(h, xd, None, False, out), iters)
        p0 = B.sconv_fc_plan(h, N)
        B.sconv_fc_tune(h, xd, out, max_plans)
        ms1 = time_gpu(lambda: B.sconv_fc_forward(h, xd, None, False, out), iters)
        p1 = B.sconv_fc_plan(h, N)
        print(f"{name} N {N}: model's choice {ms0*1e3:.1f} us, tuned {ms1*1e3:.1f} us ({100*(ms1/ms0-1):+.1f} %)"
              f"{'' if p0 == p1 else f', {p0} -> {p1}'}")
        emit(dict(report="tune", layer=name, N=N, density=dens, t_model_choice_us=ms0 * 1e3, t_tuned_us=ms1 * 1e3,
                  plan_model=p0, plan_tuned=p1))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("what", choices=["latency", "sweep", "skewed", "extra", "onebyone", "fc", "tune", "all"])
    ap.add_argument("--iters", type=int, default=20)
    args = ap.parse_args()
    if not torch.cuda.is_available():
        print("report: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.what in ("latency", "all"):
        report_latency()
    if args.what in ("sweep", "all"):
        report_sweep(args.iters)
    if args.what in ("skewed", "all"):
        report_skewed(args.iters)
    if args.what in ("extra", "all"):
        report_extra(args.iters)
    if args.what in ("onebyone", "all"):
        report_extra(args.iters, 5, "# 1x1 layers of inception modules, batch 64: Section 2.2 predicts no useful sparsity range "
                                    "when x_upper >= x_lower")
    if args.what in ("fc", "all"):
        report_fc(args.iters)
    if args.what in ("tune", "all"):
        report_tune(args.iters)
    return 0


if __name__ == "__main__":
    sys.exit(main())
