"""Oracle for the roofline performance model.  TEST INFRASTRUCTURE ONLY.

Section 2.2 written out in plain fp64 Python, in the section's order:

    t_dense          = C / F
    t_sparse_compute = alpha * x * C / F
    t_sparse_bw      = (S_A + beta * x * S_W) / B
    speedup          = t_dense / max(t_sparse_compute, t_sparse_bw)

C is the FLOP count of the dense convolution, S_A the bytes of the input and
output activations, S_W the bytes of the dense weights (all three "without
considering sparsity"), x the nonzero density, F and B the achievable FLOP/s and
memory bandwidth, alpha the compute overhead of the sparse kernel, beta the
storage overhead of its format.  The upper bound of useful sparsity is the x at
which the two sparse times are equal; the lower bound is x = 1/alpha.

Readings where the section leaves something open: C counts a multiply-add as
two FLOPs over the whole batch; S_A counts each unpadded activation once;
S_W counts each dense weight once per call.  With Table 1's F and B these
reproduce the section's own worked numbers (the pins in the tests).

Two additions, both off by default so that the four formulas above stay as printed:

* lowered=True models the comparison the section's figure draws ("conv5 lowered"): sparse convolution on
  tensors lowered to matrices.  Lowering replicates the input (Section 2.1), so the activation bytes
  become those of the lowered matrix, C*R*S rows by OH*OW columns per image, plus the output.  Creating
  that matrix is not charged (the paper leaves the cost of lowering out of its dense proxy as well).
* t_fixed is a per-call time (launch, prologue, epilogue) added to the sparse time.  It is not in the paper;
  it is 0 unless a measured value is passed in.

When alpha is not given it is derived for a machine whose sparse kernel is
limited by either its vector multiply-add rate or the bandwidth of the on-chip
memory its operands are read from:

    F_sparse = lane_efficiency * min(fma_flops, 2 * lds_bytes_per_s / lds_bytes_per_fma)
    alpha    = F / F_sparse
"""
from __future__ import annotations

import math


def layer_counts(layer, N: int, lowered: bool = False):
    Cg = layer.C // layer.groups
    OH = (layer.H + 2 * layer.pad - layer.R) // layer.stride + 1
    OW = (layer.W + 2 * layer.pad - layer.S) // layer.stride + 1
    flops = 2.0 * layer.K * Cg * layer.R * layer.S * OH * OW * N
    in_elems = layer.C * layer.R * layer.S * OH * OW if lowered else layer.C * layer.H * layer.W
    s_a = 4.0 * N * (in_elems + layer.K * OH * OW)
    s_w = 4.0 * layer.K * Cg * layer.R * layer.S
    return flops, s_a, s_w


def derive_alpha(F, fma_flops, lds_bytes_per_s, lds_bytes_per_fma, lane_efficiency):
    f_sparse = lane_efficiency * min(fma_flops, 2.0 * lds_bytes_per_s / lds_bytes_per_fma)
    return F / f_sparse


def predict(layer, N: int, x: float, F: float, B: float, alpha: float, beta: float = 2.0,
            lowered: bool = False, t_fixed: float = 0.0):
    flops, s_a, s_w = layer_counts(layer, N, lowered)
    t_dense = flops / F
    t_sc = alpha * x * flops / F
    t_sbw = (s_a + beta * x * s_w) / B
    t_sparse = t_fixed + max(t_sc, t_sbw)
    # density at which compute time equals bandwidth time
    denom = alpha * flops / F - beta * s_w / B
    x_upper = (s_a / B) / denom if denom > 0 else math.inf
    return {
        "flops_dense": flops,
        "bytes_act": s_a,
        "bytes_w": s_w,
        "alpha": alpha,
        "t_dense": t_dense,
        "t_sparse_compute": t_sc,
        "t_sparse_bw": t_sbw,
        "t_sparse": t_sparse,
        "speedup": t_dense / t_sparse,
        "effective_flops": flops / t_sparse,
        "actual_flops": x * flops / t_sparse,
        "x_upper": x_upper,
        "x_lower": 1.0 / alpha,
        "bandwidth_bound": t_sbw > t_sc,
    }


def gsl_decide(layer, N: int, x: float, stabilized: bool, F: float, B: float, alpha: float, beta: float = 2.0) -> str:
    """Section 2.3, the algorithm's per-layer rules, with sparsity bounds written as densities:
    initialise: a layer without speedup potential (empty useful range) is excluded;
    periodically: sparsity >= upper bound of the useful range -> stop pruning;
                  stabilised sparsity <= lower bound          -> stop and restore the dense weights;
    otherwise the layer stays in the pruning set."""
    p = predict(layer, N, x, F, B, alpha, beta)
    if not p["x_upper"] < p["x_lower"]:
        return "exclude"
    if x <= p["x_upper"]:
        return "stop"
    if stabilized and x >= p["x_lower"]:
        return "restore_dense"
    return "prune"
