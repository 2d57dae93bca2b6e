"""CPU oracle of the fully connected path: sparse weights times dense activations.  TEST INFRASTRUCTURE ONLY.

The paper treats a pruned fully connected layer as a sparse-matrix x dense-matrix product (end of
Section 2.1).  Its result has a plain definition, the matrix product with the pruned weights set to zero,
so the oracle is that definition in fp64 with numpy's matmul as the one library step.  Only tests, the
smoke check and the benchmark's cpu_baseline leg may import this; it shares nothing with the HIP package.
"""
from __future__ import annotations

import numpy as np


def spmdm(w: np.ndarray, x_t: np.ndarray):
    """w: pruned weights [K][C] (zeros = pruned), x_t: activations [C][N], feature-major.
    Returns (out_t [K][N] in fp64, absum [K][N] = sum over c of |w[k][c] * x_t[c][n]|)."""
    W = np.asarray(w, dtype=np.float64).reshape(w.shape[0], -1)
    X = np.asarray(x_t, dtype=np.float64)
    assert W.shape[1] == X.shape[0]
    return W @ X, np.abs(W) @ np.abs(X)


def bias_relu_t(out_t: np.ndarray, absum: np.ndarray, bias, relu: bool):
    """out_t + bias[k] per row, then max(., 0); returns (result, scale of the fp32 tolerance)."""
    res = np.array(out_t, dtype=np.float64, copy=True)
    scale = np.array(absum, dtype=np.float64, copy=True)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64).reshape(-1, 1)
        res += b
        scale += np.abs(b)
    if relu:
        res = np.where(res > 0, res, 0.0)
    return res, scale
