#!/usr/bin/env python3
"""A workload for rocprofv3: the layers of one benchmark configuration, launched round-robin through the
C-ABI library exactly as bench.py launches conv2-5, with a log of which launch belongs to which layer.

    rocprofv3 ... -- python3 -m paper_1608_01409_amd.profile_run CONFIG [--steps K] [--warmup W] [--copy-probe-mb M] [--log PATH]

CONFIG: latency (conv3, batch 1), alexnet (conv2-5, batch 256, density 0.10: bench.py's step), skewed (conv3 / conv4
with power-law rows, batch 256), goog (3x3, 5x5 and the strided conv1, batch 64), onebyone (1x1 layers, batch 64),
fc (AlexNet's fully connected layers as sparse x dense products).  The log (JSON, default profile_run_log.json in the
current directory) lists, in launch order, the layer of every forward call and how many kernels it launches
(1, plus 1 for the reduction of a channel-split tiling, plus 1 for the phase images of a strided layer);
profile_summary.py uses it to attribute the profiler's dispatches.  Inputs are the seeded synthetic ones of
workloads.py; the tilings are the cost model's (nothing is timed or tuned here, so every dispatch is in the log).
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np
import torch

from . import binding as B
from . import workloads as wl


def conv_layers(cfg_index, cases, skewed=False):
    out = []
    for li, (name, N, dens) in enumerate(cases):
        layer = wl.LAYERS[name]
        x, w = wl.make_case(cfg_index, li, layer, N, dens, skewed=skewed)
        h = B.sconv_create_csr(layer, w)
        xd = torch.from_numpy(x).cuda()
        o = torch.empty((N, layer.K, layer.OH, layer.OW), dtype=torch.float32, device="cuda")
        B.sconv_forward(h, xd, o)                      # settles the tiling for this batch size
        plan = B.sconv_csr_info(h)["plan"]
        kernels = 1 + (1 if plan["splits"] > 1 else 0) + (1 if layer.stride > 1 and not (plan["kernel"] == 2 or (layer.pad == 0 and plan["kernel"] in (3, 4))) else 0)
        nnz = B.sconv_csr_info(h)["nnz"]
        out.append(dict(name=name, run=(lambda h=h, xd=xd, o=o: B.sconv_forward(h, xd, o)), kernels=kernels, plan=plan, N=N,
                        flops=2.0 * nnz * layer.OH * layer.OW * N,
                        bytes=4.0 * N * (layer.C * layer.H * layer.W + layer.K * layer.OH * layer.OW) + 8.0 * nnz))
    return out


def fc_layers():
    out = []
    for i, (name, N, dens) in enumerate(wl.FC_CONFIG):
        C_in, K = wl.FC_LAYERS[name]
        x_t, w = wl.make_fc_case(i, name, N, dens)
        h = B.sconv_create_csr(B.fc_layer(C_in, K), w.reshape(K, C_in, 1, 1), dict(kernel=2))
        xd = torch.from_numpy(x_t).cuda()
        o = torch.empty((K, N), dtype=torch.float32, device="cuda")
        B.sconv_fc_forward(h, xd, None, False, o)
        plan = B.sconv_fc_plan(h, N)
        nnz = int(np.count_nonzero(w))
        out.append(dict(name=f"{name}@{N}", run=(lambda h=h, xd=xd, o=o: B.sconv_fc_forward(h, xd, None, False, o)),
                        kernels=1 + (1 if plan["splits"] > 1 else 0), plan=plan, N=N, flops=2.0 * nnz * N,
                        bytes=4.0 * N * (C_in + K) + 8.0 * nnz))
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("config", choices=["latency", "alexnet", "skewed", "goog", "onebyone", "fc"])
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--copy-probe-mb", type=int, default=0)
    ap.add_argument("--log", default="profile_run_log.json")
    args = ap.parse_args()
    torch.cuda.set_device(0)
    if args.config == "latency":
        layers = conv_layers(0, wl.CONFIGS[0])
    elif args.config == "alexnet":
        layers = conv_layers(1, wl.CONFIGS[1])
    elif args.config == "skewed":
        layers = conv_layers(3, [("conv3", 256, 0.10), ("conv4", 256, 0.10)], skewed=True)
    elif args.config == "goog":
        layers = conv_layers(4, wl.CONFIGS[4])
    elif args.config == "onebyone":
        layers = conv_layers(5, wl.CONFIGS[5])
    else:
        layers = fc_layers()
    torch.cuda.synchronize()
    calls = [dict(layer=L["name"], kernels=L["kernels"], phase="setup") for L in layers]   # the settling calls above
    for phase, n in (("warmup", args.warmup), ("timed", args.steps)):
        if phase == "timed" and args.copy_probe_mb:
            src = torch.empty(args.copy_probe_mb * 2 ** 20 // 4, dtype=torch.float32, device="cuda").normal_()
            dst = torch.empty_like(src)
            dst.copy_(src)
            torch.cuda.synchronize()
        for _ in range(n):
            for L in layers:
                L["run"]()
                calls.append(dict(layer=L["name"], kernels=L["kernels"], phase=phase))
    torch.cuda.synchronize()
    json.dump(dict(config=args.config, copy_probe_mb=args.copy_probe_mb,
                   layers=[dict(name=L["name"], plan=L["plan"], N=L["N"], flops=L["flops"], bytes=L["bytes"], kernels=L["kernels"])
                           for L in layers], calls=calls), open(args.log, "w"))
    return 0


if __name__ == "__main__":
    sys.exit(main())
