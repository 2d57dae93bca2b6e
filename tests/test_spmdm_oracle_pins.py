"""Pins of the fully connected (sparse x dense) oracle: brute force, a sparse-matrix library, the
convolution oracle on 1x1 images, and planted mistakes."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle import spmdm_oracle as so
from paper_1608_01409_amd import workloads as wl


def case(K, C, N, density, seed):
    rng = np.random.default_rng(seed)
    w = np.where(rng.random((K, C)) < density, rng.standard_normal((K, C)), 0).astype(np.float32)
    x_t = rng.standard_normal((C, N)).astype(np.float32)
    return w, x_t


def test_brute_force_on_tiny_inputs():
    w, x_t = case(5, 7, 4, 0.5, 1)
    out, ab = so.spmdm(w, x_t)
    for k in range(5):
        for n in range(4):
            acc = 0.0
            aab = 0.0
            for c in range(7):
                acc += float(w[k, c]) * float(x_t[c, n])
                aab += abs(float(w[k, c]) * float(x_t[c, n]))
            assert abs(out[k, n] - acc) <= 1e-14 * max(aab, 1.0)
            assert abs(ab[k, n] - aab) <= 1e-14 * max(aab, 1.0)


def test_equals_sparse_library_product():
    w, x_t = case(60, 90, 12, 0.1, 2)
    out, _ = so.spmdm(w, x_t)
    ref = sp.csr_matrix(w.astype(np.float64)) @ x_t.astype(np.float64)
    assert np.allclose(out, ref, rtol=0, atol=1e-12)


def test_equals_convolution_oracle_on_one_by_one_images(oracle):
    K, C, N = 9, 14, 8
    w, x_t = case(K, C, N, 0.3, 3)
    layer = wl.Layer("fc", C, 1, 1, K, 1, 1, 1, 0, 1)
    x = np.ascontiguousarray(x_t.T).reshape(N, C, 1, 1)
    ref, ab, _ = oracle.sparse_conv(layer, w.reshape(K, C, 1, 1), x)
    out, ab2 = so.spmdm(w, x_t)
    assert np.allclose(out, ref.reshape(N, K).T, rtol=0, atol=1e-13)
    assert np.allclose(ab2, ab.reshape(N, K).T, rtol=0, atol=1e-13)


def test_zero_rows_and_identity():
    w = np.zeros((4, 4), dtype=np.float32)
    w[[0, 1, 3], [0, 1, 3]] = 1
    x_t = np.arange(12, dtype=np.float32).reshape(4, 3)
    out, ab = so.spmdm(w, x_t)
    assert np.array_equal(out[[0, 1, 3]], x_t[[0, 1, 3]].astype(np.float64))
    assert np.all(out[2] == 0) and np.all(ab[2] == 0)


def test_planted_mistakes_are_caught():
    w, x_t = case(6, 6, 6, 0.6, 4)
    out, _ = so.spmdm(w, x_t)
    assert not np.allclose(out, (w.astype(np.float64).T @ x_t.astype(np.float64)))          # transposed weights
    assert not np.allclose(out, (x_t.astype(np.float64).T @ w.astype(np.float64).T).T[::-1])  # reversed rows


def test_bias_relu_rows():
    w, x_t = case(5, 8, 4, 0.5, 5)
    out, ab = so.spmdm(w, x_t)
    bias = np.array([10, -10, 0.5, -0.5, 0], dtype=np.float32)
    res, scale = so.bias_relu_t(out, ab, bias, True)
    assert np.allclose(res, np.maximum(out + bias[:, None].astype(np.float64), 0))
    assert np.all(res[1] == 0) and np.all(res[0] > 0)
    assert np.allclose(scale, ab + np.abs(bias)[:, None])
    res2, scale2 = so.bias_relu_t(out, ab, None, False)
    assert np.array_equal(res2, out) and np.array_equal(scale2, ab)


def test_fully_connected_layer_with_bias_and_relu_is_torchs_linear():
    """The whole fully connected oracle (product, bias per output feature, ReLU) against the library's own
    fp64 layer: torch.nn.functional.linear takes image-major activations [N][C] and returns [N][K]."""
    import torch

    w, x_t = case(9, 14, 6, 0.4, 6)
    bias = np.linspace(-0.3, 0.3, 9).astype(np.float32)
    out, ab = so.spmdm(w, x_t)
    res, _ = so.bias_relu_t(out, ab, bias, True)
    lin = torch.nn.functional.linear(torch.from_numpy(x_t.T.astype(np.float64)), torch.from_numpy(w.astype(np.float64)),
                                     torch.from_numpy(bias.astype(np.float64)))
    want = torch.relu(lin).numpy().T
    assert (want == 0).any() and (want > 0).any()
    assert np.allclose(res, want, rtol=1e-13, atol=1e-15)
    # a bias on the wrong axis, or a ReLU before the bias, does not survive this
    assert not np.allclose(np.maximum(out, 0) + bias[:, None], want)
    res_nb, _ = so.bias_relu_t(out, ab, None, True)
    assert np.allclose(res_nb, torch.relu(lin - torch.from_numpy(bias.astype(np.float64))).numpy().T, rtol=1e-13, atol=1e-15)
