#!/usr/bin/env python3
"""Benchmark of the direct-sparse-convolution hot path on one MI355X.

A step is one forward pass of AlexNet conv2, conv3, conv4 and conv5 (batch 256,
10 % nonzero density, seeded synthetic weights and activations already resident
in HBM) through the C-ABI library.  The metric is the rate of useful
multiply-adds, 2*nnz*OH*OW*N FLOP per layer (nonzeros only; the paper calls
this the actual FLOP/s, Section 3.2), summed over the four layers and divided
by the wall time of the step.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# plain v_fma_f32: 256 CUs x 4 SIMDs x 16 lanes x 2 FLOP x 2.4 GHz (packed FP32 would double it)
PEAK_FMA_TFLOPS = 78.6
PEAK_FP32_PUBLISHED_TFLOPS = 157.3


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tune", type=int, default=8,
                    help="during set-up let sconv_tune time this many candidate tilings per layer and keep the "
                         "fastest, as a deployment of the library would (0: the cost model's choice, untimed)")
    ap.add_argument("--layer-events-every", type=int, default=4,
                    help="time the individual kernels (an event pair around each) on every M-th timed step; the pairs "
                         "cost stream time, so M = 1 lengthens every step by a few percent")
    ap.add_argument("--copy-probe-mb", type=int, default=0,
                    help="also launch one plain device copy of this many MiB (a known-size reference for "
                         "scaling the HBM byte counters of a profiler run)")
    ap.add_argument("--dispatch-log", default="",
                    help="write the order of the forward calls of the warm-up and timed steps here (JSON), for "
                         "profile_summary.py to attribute a profiler's dispatches to layers")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path shards over the batch with no exchange "
              "between GPUs, so more GPUs add nothing to measure); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1608_01409_amd import binding as B
    from paper_1608_01409_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    layers = []
    for li, (name, N, dens) in enumerate(wl.CONFIGS[1]):
        layer = wl.LAYERS[name]
        x, w = wl.make_case(1, li, layer, N, dens)
        h = B.sconv_create_csr(layer, w)
        info = B.sconv_csr_info(h)
        xd = torch.from_numpy(x).cuda()
        out = torch.empty((N, layer.K, info["OH"], info["OW"]), dtype=torch.float32, device="cuda")
        if args.tune > 0:
            B.sconv_tune(h, xd, out, max_plans=args.tune, stream=stream)
        flops = 2.0 * info["nnz"] * info["OH"] * info["OW"] * N
        dense_flops = 2.0 * layer.K * layer.Cg * layer.R * layer.S * info["OH"] * info["OW"] * N
        layers.append(dict(name=name, layer=layer, N=N, h=h, x=xd, out=out, flops=flops, dense_flops=dense_flops,
                           plan=info["plan"], nnz=info["nnz"], host=(x, w)))

    def step(events=None):
        for i, L in enumerate(layers):
            if events is not None:
                events[i][0].record(stream)
            B.sconv_forward(L["h"], L["x"], L["out"], stream=stream)
            if events is not None:
                events[i][1].record(stream)

    # events first: nothing but the warm-up steps themselves runs between set-up and the timed steps.  An event pair
    # around a kernel keeps the next launch from starting behind it (~3 us of stream time per pair: on every step that
    # is 3.5 % of the step), so the kernels are timed on every M-th timed step only; every step gets one event at its start.
    every = max(1, args.layer_events_every)
    timed_steps = [k for k in range(args.steps) if k % every == 0]
    ev = {k: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in layers] for k in timed_steps}
    step_ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.copy_probe_mb:
        src = torch.empty(args.copy_probe_mb * 2 ** 20 // 4, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
    for L in layers:  # the tiling follows the batch size at the first call
        L["plan"] = B.sconv_csr_info(L["h"])["plan"]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step_ev[k].record(stream)
        step(ev.get(k))
    step_ev[args.steps].record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if args.dispatch_log:
        def n_kernels(L):
            return 1 + (1 if L["plan"]["splits"] > 1 else 0) + (1 if L["layer"].stride > 1 and not (L["plan"]["kernel"] == 2 or (L["layer"].pad == 0 and L["plan"]["kernel"] in (3, 4))) else 0)
        calls = [dict(layer=L["name"], kernels=n_kernels(L), phase=ph) for ph, n in (("warmup", args.warmup), ("timed", args.steps))
                 for _ in range(n) for L in layers]
        json.dump(dict(config="bench.py: AlexNet conv2-5, batch 256, density 0.10" + (f", tilings tuned (--tune {args.tune})" if args.tune > 0 else ""),
                       copy_probe_mb=args.copy_probe_mb,
                       layers=[dict(name=L["name"], plan=L["plan"], N=L["N"], flops=L["flops"], kernels=n_kernels(L),
                                    bytes=4.0 * L["N"] * (L["layer"].C * L["layer"].H * L["layer"].W + L["layer"].K * L["layer"].OH * L["layer"].OW) + 8.0 * L["nnz"])
                               for L in layers], calls=calls), open(args.dispatch_log, "w"))
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    total_flops = sum(L["flops"] for L in layers)
    value = total_flops / (ms_per_step * 1e-3) / 1e9

    per_layer = []
    for i, L in enumerate(layers):
        ms = float(np.mean([ev[k][i][0].elapsed_time(ev[k][i][1]) for k in timed_steps]))
        tf = L["flops"] / (ms * 1e-3) / 1e12
        per_layer.append(dict(layer=L["name"], kernel_us=round(ms * 1e3, 2), tflops=round(tf, 3),
                              effective_tflops=round(L["dense_flops"] / (ms * 1e-3) / 1e12, 2),
                              frac_of_fma_peak=round(tf / PEAK_FMA_TFLOPS, 4), nnz=L["nnz"], plan=L["plan"]))
    # The target is per layer, so the headline fraction is the LOWEST of the four layers, not the one of the
    # longest-running (and most efficient) kernel; that one is listed beside it.
    low = min(range(len(layers)), key=lambda i: per_layer[i]["tflops"])
    dom = max(range(len(layers)), key=lambda i: per_layer[i]["kernel_us"])
    achieved = per_layer[low]["tflops"]
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(layers[low]["name"], {}).get("bytes")
            traffic_source = ("profiles/hbm_traffic.json: rocprofv3 FETCH_SIZE + WRITE_SIZE per launch from an earlier "
                              "profiler run of this command, stored; not measured in this run")
        except (OSError, ValueError):
            traffic = None

    def kname(i):
        return ("sconv_lds2_kernel" if layers[i]["plan"]["kernel"] in (3, 4) else "sconv_lds_kernel") + f" on {layers[i]['name']}"

    roofline = dict(bound="alu", achieved=achieved, peak=PEAK_FMA_TFLOPS, unit="TFLOP/s",
                    frac=round(achieved / PEAK_FMA_TFLOPS, 4), traffic=traffic, traffic_source=traffic_source,
                    kernel=kname(low) + " (the lowest fraction of the four layers)",
                    longest_kernel=dict(kernel=kname(dom), achieved=per_layer[dom]["tflops"],
                                        frac=per_layer[dom]["frac_of_fma_peak"]),
                    frac_of_published_fp32_vector=round(achieved / PEAK_FP32_PUBLISHED_TFLOPS, 4),
                    step_frac=round(value / 1e3 / PEAK_FMA_TFLOPS, 4), per_layer=per_layer)

    # how steady the timed region was: the GPU's power management settles over the first tens of milliseconds
    # of load, and steps taken during that time run up to 15 % slower than later ones
    step_us = [step_ev[k].elapsed_time(step_ev[k + 1]) * 1e3 for k in range(args.steps)]
    q = max(1, args.steps // 4)
    steadiness = dict(first_quarter_us=round(float(np.mean(step_us[:q])), 1), last_quarter_us=round(float(np.mean(step_us[-q:])), 1))

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import sconv_oracle as O
        t_cpu, used, reps = 0.0, 0, 0
        csr = []
        checked = []
        for L in layers:
            x, w = L["host"]
            rp, ci, v = O.csr_from_dense(L["layer"], w)
            csr.append((rp, O.lower_offsets(L["layer"], rp, ci), v))
            # what the timed steps left in the output buffers, against the fp64 oracle on sampled images
            idx = sorted({0, L["N"] // 3, (2 * L["N"]) // 3, L["N"] - 1})
            ref, ab = O.forward_f64(L["layer"], rp, csr[-1][1], v, x[idx])
            got = L["out"][idx].cpu().numpy().astype(np.float64)
            if not np.all(np.abs(got - ref) <= 1e-5 * ab):
                print(f"bench.py: {L['name']} does not match the oracle with tiling {L['plan']}", file=sys.stderr)
                return 3
            checked.append(f"{L['name']}: images {idx}")
        while t_cpu < 10.0 and reps < 20:
            for L, (rp, off, v) in zip(layers, csr):
                a = time.perf_counter()
                _, used = O.forward_f32(L["layer"], rp, off, v, L["host"][0])
                t_cpu += time.perf_counter() - a
            reps += 1
        cpu = dict(value=round(total_flops * reps / t_cpu / 1e9, 2), unit="GFLOP/s", cores=used, kind="oracle",
                   sample=f"the whole step (conv2-5, batch 256) x {reps} repetitions, fp32 loop of Figure 2, OpenMP",
                   gpu_outputs_checked="the timed steps' outputs within 1e-5 * sum|w*x| of the fp64 oracle on " + "; ".join(checked))

    print(json.dumps({
        "metric": "effective GFLOP/s (2*nnz*OH*OW*N/s), AlexNet conv2-5 @ 10% density",
        "value": round(value, 1), "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "AlexNet conv2-conv5, batch 256, fp32, Bernoulli masks at density 0.10", "global_batch": 256,
                   "tiling": f"fastest of {args.tune} candidates timed during set-up (sconv_tune)" if args.tune > 0 else "cost model",
                   "timed_region": steadiness,
                   "kernel_timing": f"HIP event pairs around every kernel on timed steps {timed_steps[:3]}... ({len(timed_steps)} of {args.steps})",
                   "dense_equivalent_gflops": round(sum(L["dense_flops"] for L in layers) / (ms_per_step * 1e-3) / 1e9, 1)},
        "roofline": roofline, "cpu_baseline": cpu}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
