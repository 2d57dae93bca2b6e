"""Seeded synthetic layers and activations for direct sparse convolution.

This module only draws random numbers and names layer shapes.  It holds none of
the method's arithmetic (no CSR building, no offset lowering, no convolution):
the CPU oracle and the HIP library each do those on their own.  Both are handed
the same numpy arrays produced here.

The shapes are the AlexNet conv1-5 and GoogLeNet-inception-like layers the
paper evaluates (Section 3.2, Figure 5); the paper's really-pruned weight
matrices are not available, so Bernoulli masks (and a skewed, clustered
generator standing in for guided-pruning structure) are used instead.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict

import numpy as np

BASE_SEED = 160801409 * 10


@dataclass(frozen=True)
class Layer:
    """One convolution layer: C x H x W input, K filters of (C/groups) x R x S."""

    name: str
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int
    pad: int
    groups: int

    @property
    def Cg(self) -> int:
        return self.C // self.groups

    @property
    def Kg(self) -> int:
        return self.K // self.groups

    @property
    def OH(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def OW(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    def dims(self) -> dict:
        d = asdict(self)
        d.pop("name")
        return d


LAYERS = {
    "conv1": Layer("conv1", 3, 227, 227, 96, 11, 11, 4, 0, 1),
    "conv2": Layer("conv2", 96, 27, 27, 256, 5, 5, 1, 2, 2),
    "conv3": Layer("conv3", 256, 13, 13, 384, 3, 3, 1, 1, 1),
    "conv4": Layer("conv4", 384, 13, 13, 384, 3, 3, 1, 1, 2),
    "conv5": Layer("conv5", 384, 13, 13, 256, 3, 3, 1, 1, 2),
    "goog3x3": Layer("goog3x3", 192, 28, 28, 128, 3, 3, 1, 1, 1),
    "goog5x5": Layer("goog5x5", 32, 28, 28, 96, 5, 5, 1, 2, 1),
    # 1x1 "reduce" layers of inception modules: few FLOPs per activation byte, the layers for which
    # Section 2.2 predicts no useful sparsity range
    "goog1x1_reduce": Layer("goog1x1_reduce", 480, 14, 14, 16, 1, 1, 1, 0, 1),
    "goog1x1": Layer("goog1x1", 192, 28, 28, 64, 1, 1, 1, 0, 1),
}

# (layer name, batch, density) per benchmark configuration.
CONFIGS = {
    0: [("conv3", 1, 0.10)],
    1: [("conv2", 256, 0.10), ("conv3", 256, 0.10), ("conv4", 256, 0.10), ("conv5", 256, 0.10)],
    4: [("goog3x3", 64, 0.20), ("goog5x5", 64, 0.30), ("conv1", 64, 0.30)],
    5: [("goog1x1_reduce", 64, 0.30), ("goog1x1", 64, 0.30)],   # beyond the benchmark configurations
}
# Fully connected layers of AlexNet (input features, output features), batch, density: the sparse x dense
# products the paper's discussion of fully connected layers is about (end of Section 2.1).
FC_LAYERS = {"fc6": (9216, 4096), "fc7": (4096, 4096), "fc8": (4096, 1000)}
FC_CONFIG = [("fc6", 256, 0.10), ("fc7", 256, 0.10), ("fc8", 256, 0.25), ("fc7", 1024, 0.10)]


def make_fc_case(index: int, name: str, N: int, density: float):
    """(x_t [C][N] feature-major activations, w [K][C] pruned weights), seeded like make_case."""
    C_in, K = FC_LAYERS[name]
    rng_x, rng_m, rng_v = _streams(6, index)
    x_t = rng_x.standard_normal((C_in, N), dtype=np.float32)
    w = (rng_v.standard_normal((K, C_in), dtype=np.float32) * np.float32(WEIGHT_STD))
    if density < 1.0:
        w = np.where(rng_m.random((K, C_in)) < density, w, np.float32(0)).astype(np.float32)
    return x_t, w


SWEEP_DENSITIES = (0.01, 0.02, 0.05, 0.1, 0.2, 0.3, 0.5, 1.0)
WEIGHT_STD = 0.01


def _streams(cfg_index: int, layer_index: int):
    """Independent child streams in the fixed order input, mask, values."""
    ss = np.random.SeedSequence([BASE_SEED + cfg_index, layer_index])
    return [np.random.Generator(np.random.PCG64(s)) for s in ss.spawn(3)]


def make_input(rng: np.random.Generator, layer: Layer, N: int) -> np.ndarray:
    """Activations [N][C][H][W], i.i.d. standard normal, fp32."""
    return rng.standard_normal((N, layer.C, layer.H, layer.W), dtype=np.float32)


def make_uniform_weights(rng_mask, rng_val, layer: Layer, density: float) -> np.ndarray:
    """Dense-shaped pruned weights [K][C/groups][R][S]: i.i.d. Bernoulli(density)
    mask (all ones at density 1), surviving values N(0, WEIGHT_STD^2); pruned = 0."""
    shape = (layer.K, layer.Cg, layer.R, layer.S)
    vals = (rng_val.standard_normal(shape, dtype=np.float32) * np.float32(WEIGHT_STD)).astype(np.float32)
    # a drawn value of exactly 0 would silently change the pattern; nudge it.
    vals[vals == 0] = np.float32(WEIGHT_STD)
    if density >= 1.0:
        return vals
    mask = rng_mask.random(shape) < density
    return np.where(mask, vals, np.float32(0)).astype(np.float32)


def make_skewed_weights(rng_mask, rng_val, layer: Layer, mean_density: float = 0.10,
                        max_density: float = 0.60, empty_frac: float = 0.20,
                        pareto_a: float = 2.0, cluster: str = "channels") -> np.ndarray:
    """Guided-pruning-like structure: `empty_frac` of the output channels fully
    pruned, the others with a power-law density (capped at `max_density`,
    overall mean `mean_density`).  Where a row's nonzeros go:

    cluster="channels"   into a subset of active input channels (each active with
                         probability p = min(1, 2 d)), positions inside an active
                         channel kept independently with probability d / p;
    cluster="positions"  same active channels, but inside each the surviving kernel
                         positions are one contiguous run in (r, s) raster order
                         (random start, expected length d / p of the R*S positions),
                         so the kernel positions of a channel are clustered."""
    assert cluster in ("channels", "positions")
    K, Cg, R, S = layer.K, layer.Cg, layer.R, layer.S
    n_empty = int(round(empty_frac * K))
    empty = np.zeros(K, dtype=bool)
    empty[rng_mask.choice(K, size=n_empty, replace=False)] = True
    u = rng_mask.random(K)
    u = np.maximum(u, 1e-12)

    def densities(dmin):
        d = np.minimum(max_density, dmin * u ** (-1.0 / pareto_a))
        d[empty] = 0.0
        return d

    lo, hi = 0.0, max_density
    for _ in range(80):
        mid = 0.5 * (lo + hi)
        if densities(mid).mean() < mean_density:
            lo = mid
        else:
            hi = mid
    d = densities(0.5 * (lo + hi))
    vals = (rng_val.standard_normal((K, Cg, R, S), dtype=np.float32) * np.float32(WEIGHT_STD)).astype(np.float32)
    vals[vals == 0] = np.float32(WEIGHT_STD)
    w = np.zeros((K, Cg, R, S), dtype=np.float32)
    npos = R * S
    for k in range(K):
        if d[k] <= 0:
            continue
        p = min(1.0, 2.0 * d[k])
        q = d[k] / p
        active = rng_mask.random(Cg) < p
        if cluster == "channels":
            m = (rng_mask.random((Cg, R, S)) < q) & active[:, None, None]
        else:
            length = np.floor(q * npos + rng_mask.random(Cg)).astype(np.int64)      # expected q * npos
            start = np.floor(rng_mask.random(Cg) * (npos - length + 1)).astype(np.int64)
            pos = np.arange(npos)[None, :]
            m = ((pos >= start[:, None]) & (pos < (start + length)[:, None]) & active[:, None]).reshape(Cg, R, S)
        w[k] = np.where(m, vals[k], np.float32(0))
    return w


def make_case(cfg_index: int, layer_index: int, layer: Layer, N: int, density: float,
              skewed: bool = False, cluster: str = "channels"):
    """(input [N,C,H,W] fp32, weights [K,Cg,R,S] fp32 with zeros where pruned)."""
    r_in, r_mask, r_val = _streams(cfg_index, layer_index)
    x = make_input(r_in, layer, N)
    if skewed:
        w = make_skewed_weights(r_mask, r_val, layer, mean_density=density, cluster=cluster)
    else:
        w = make_uniform_weights(r_mask, r_val, layer, density)
    return x, w


def small_layer(name="tiny", **kw) -> Layer:
    base = dict(C=4, H=6, W=7, K=6, R=3, S=2, stride=1, pad=1, groups=1)
    base.update(kw)
    return Layer(name, **base)
