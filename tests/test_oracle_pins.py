"""Pins for the CPU oracle: everything here checks the oracle against something
that is not the oracle (Eq. (1) written out by brute force, a library dense
convolution, closed forms, invariants).  No GPU, no HIP library."""
import itertools

import numpy as np
import pytest
import torch

from paper_1608_01409_amd import workloads as wl


# ---------------------------------------------------------------- brute force
def brute_force_conv(layer, w, x):
    """Eq. (1) of Section 2.1 as seven nested loops over the UNPADDED input with
    bounds checks (so it shares neither the padded copy nor the offset formula
    with the oracle).  fp64.  Also returns the sum of |products|."""
    N = x.shape[0]
    Cg, Kg = layer.C // layer.groups, layer.K // layer.groups
    OH = (layer.H + 2 * layer.pad - layer.R) // layer.stride + 1
    OW = (layer.W + 2 * layer.pad - layer.S) // layer.stride + 1
    out = np.zeros((N, layer.K, OH, OW))
    ab = np.zeros_like(out)
    for n, k, y, xx in itertools.product(range(N), range(layer.K), range(OH), range(OW)):
        g = k // Kg
        acc = 0.0
        a = 0.0
        for c in range(Cg):
            for r in range(layer.R):
                iy = y * layer.stride + r - layer.pad
                if iy < 0 or iy >= layer.H:
                    continue
                for s in range(layer.S):
                    ix = xx * layer.stride + s - layer.pad
                    if ix < 0 or ix >= layer.W:
                        continue
                    p = float(w[k, c, r, s]) * float(x[n, g * Cg + c, iy, ix])
                    acc += p
                    a += abs(p)
        out[n, k, y, xx] = acc
        ab[n, k, y, xx] = a
    return out, ab


def rand_case(layer, N, density, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, layer.C, layer.H, layer.W)).astype(np.float32)
    w = rng.standard_normal((layer.K, layer.Cg, layer.R, layer.S)).astype(np.float32)
    if density < 1:
        w = np.where(rng.random(w.shape) < density, w, np.float32(0)).astype(np.float32)
    return x, w


TINY = [
    dict(C=4, H=6, W=7, K=6, R=3, S=2, stride=1, pad=1, groups=1),
    dict(C=4, H=6, W=7, K=6, R=3, S=2, stride=1, pad=1, groups=2),
    dict(C=2, H=5, W=5, K=4, R=3, S=3, stride=1, pad=0, groups=1),
    dict(C=4, H=7, W=6, K=4, R=2, S=3, stride=2, pad=1, groups=2),
    dict(C=3, H=9, W=11, K=3, R=3, S=5, stride=2, pad=2, groups=1),
    dict(C=2, H=13, W=12, K=2, R=5, S=4, stride=4, pad=0, groups=1),
    dict(C=6, H=4, W=4, K=6, R=1, S=1, stride=1, pad=0, groups=3),
    dict(C=2, H=8, W=9, K=4, R=3, S=3, stride=4, pad=2, groups=2),
    dict(C=2, H=6, W=10, K=2, R=3, S=3, stride=3, pad=1, groups=1),  # trailing rows/cols ignored
]


@pytest.mark.parametrize("dims", TINY)
@pytest.mark.parametrize("N", [1, 3])
def test_oracle_matches_brute_force(oracle, dims, N):
    layer = wl.small_layer(**dims)
    x, w = rand_case(layer, N, 0.4, seed=hash(tuple(dims.values())) % 1000 + N)
    out, ab, _ = oracle.sparse_conv(layer, w, x)
    ref, ref_ab = brute_force_conv(layer, w, x)
    assert out.shape == ref.shape
    assert np.all(np.abs(out - ref) <= 1e-12 * ref_ab + 1e-300)
    assert np.all(np.abs(ab - ref_ab) <= 1e-12 * ref_ab + 1e-300)


# ------------------------------------------------ density 1 == dense library conv
@pytest.mark.parametrize("dims", TINY + [dict(C=8, H=13, W=13, K=12, R=3, S=3, stride=1, pad=1, groups=2)])
def test_density_one_equals_library_dense_conv(oracle, dims):
    layer = wl.small_layer(**dims)
    x, w = rand_case(layer, 2, 1.0, seed=7)
    out, ab, csr = oracle.sparse_conv(layer, w, x)
    assert len(csr[3]) == w.size  # nothing dropped
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     stride=layer.stride, padding=layer.pad, groups=layer.groups).numpy()
    assert np.all(np.abs(out - ref) <= 1e-12 * ab + 1e-300)


def test_sparse_equals_library_conv_with_masked_weights(oracle):
    layer = wl.small_layer(C=16, H=13, W=13, K=24, R=3, S=3, stride=1, pad=1, groups=1)
    x, w = rand_case(layer, 3, 0.1, seed=11)
    out, ab, _ = oracle.sparse_conv(layer, w, x)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     stride=1, padding=1).numpy()
    assert np.all(np.abs(out - ref) <= 1e-12 * ab + 1e-300)


# ---------------------------------------------------------------- invariants
def test_zero_mask_gives_exact_zeros(oracle):
    layer = wl.small_layer()
    x, _ = rand_case(layer, 2, 1.0, seed=3)
    w = np.zeros((layer.K, layer.Cg, layer.R, layer.S), dtype=np.float32)
    w[0, 0, 0, 0] = -0.0  # negative zero is pruned as well
    out, ab, csr = oracle.sparse_conv(layer, w, x)
    assert len(csr[3]) == 0 and np.all(csr[0] == 0)
    assert np.all(out == 0) and np.all(ab == 0)


def test_empty_rows_are_zero_and_others_unaffected(oracle):
    layer = wl.small_layer(K=6)
    x, w = rand_case(layer, 2, 0.5, seed=5)
    w2 = w.copy()
    w2[[1, 4]] = 0
    out, _, _ = oracle.sparse_conv(layer, w, x)
    out2, _, csr = oracle.sparse_conv(layer, w2, x)
    assert csr[0][1] == csr[0][2] and csr[0][4] == csr[0][5]
    assert np.all(out2[:, [1, 4]] == 0)
    assert np.array_equal(out2[:, [0, 2, 3, 5]], out[:, [0, 2, 3, 5]])


def test_linear_in_weights(oracle):
    layer = wl.small_layer(C=4, H=8, W=8, K=5, R=3, S=3, stride=2, pad=1, groups=1)
    x, w1 = rand_case(layer, 2, 0.3, seed=21)
    _, w2 = rand_case(layer, 2, 0.3, seed=22)
    # weights on a 2^-10 grid, so that a*w1 + b*w2 is exact in fp32 where the patterns overlap
    w1 = (np.round(w1 * 1024) / 1024).astype(np.float32)
    w2 = (np.round(w2 * 1024) / 1024).astype(np.float32)
    a, b = np.float32(0.5), np.float32(-2.0)
    o1, ab1, _ = oracle.sparse_conv(layer, w1, x)
    o2, ab2, _ = oracle.sparse_conv(layer, w2, x)
    o12, _, _ = oracle.sparse_conv(layer, a * w1 + b * w2, x)
    scale = abs(a) * ab1 + abs(b) * ab2
    assert np.all(np.abs(o12 - (a * o1 + b * o2)) <= 1e-12 * scale + 1e-300)


@pytest.mark.parametrize("stride,pad", [(1, 0), (1, 2), (2, 1), (4, 0), (3, 2)])
def test_single_nonzero_is_a_shifted_window(oracle, stride, pad):
    """One weight equal to 1 at (k,c,r,s): the output plane is the strided
    window of the padded input channel starting at (r,s) -- exactly."""
    layer = wl.small_layer(C=4, H=9, W=10, K=4, R=3, S=4, stride=stride, pad=pad, groups=2)
    x, _ = rand_case(layer, 2, 1.0, seed=9)
    OH, OW = layer.OH, layer.OW
    xp = np.pad(x, ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    for (k, c, r, s) in [(0, 0, 0, 0), (1, 1, 2, 3), (2, 0, 1, 2), (3, 1, 2, 0)]:
        w = np.zeros((layer.K, layer.Cg, layer.R, layer.S), dtype=np.float32)
        w[k, c, r, s] = 1.0
        out, _, _ = oracle.sparse_conv(layer, w, x)
        g = k // layer.Kg
        win = xp[:, g * layer.Cg + c, r:r + (OH - 1) * stride + 1:stride, s:s + (OW - 1) * stride + 1:stride]
        assert np.array_equal(out[:, k], win.astype(np.float64))
        others = [kk for kk in range(layer.K) if kk != k]
        assert np.all(out[:, others] == 0)


def test_one_by_one_conv_is_a_sparse_matrix_product(oracle):
    """R=S=1, stride 1, no pad: out_n = W_(1) . in_n with W_(1) the K x C CSR matrix."""
    import scipy.sparse as sp
    layer = wl.small_layer(C=12, H=5, W=6, K=9, R=1, S=1, stride=1, pad=0, groups=1)
    x, w = rand_case(layer, 3, 0.3, seed=13)
    out, ab, (rowptr, colidx, off, val) = oracle.sparse_conv(layer, w, x)
    A = sp.csr_matrix((val.astype(np.float64), colidx, rowptr), shape=(layer.K, layer.C))
    for n in range(3):
        ref = A @ x[n].reshape(layer.C, -1).astype(np.float64)
        assert np.all(np.abs(out[n].reshape(layer.K, -1) - ref) <= 1e-12 * ab[n].reshape(layer.K, -1) + 1e-300)


# -------------------------------------------------------------- CSR + lowering
def test_csr_is_canonical_and_complete(oracle):
    layer = wl.small_layer(C=6, K=6, groups=2)
    _, w = rand_case(layer, 1, 0.3, seed=17)
    w[2, 1, 1, 1] = np.float32("nan")      # kept
    w[3, 0, 0, 0] = np.float32(1e-45)      # denormal kept
    rowptr, colidx, val = oracle.csr_from_dense(layer, w)
    flat = w.reshape(layer.K, -1)
    assert rowptr[0] == 0 and rowptr[-1] == len(val)
    for k in range(layer.K):
        cols = colidx[rowptr[k]:rowptr[k + 1]]
        expect = np.flatnonzero(~(flat[k] == 0))
        assert np.array_equal(cols, expect)
        assert np.array_equal(val[rowptr[k]:rowptr[k + 1]].view(np.uint32), flat[k, expect].view(np.uint32))


@pytest.mark.parametrize("dims", TINY)
def test_lowered_offsets_closed_form_and_additivity(oracle, dims):
    """off = f(c,r,s) on the padded image, and off + f(0, y*stride, x*stride)
    = f(c, y*stride + r, x*stride + s): the additivity Section 2.1 assumes."""
    layer = wl.small_layer(**dims)
    _, w = rand_case(layer, 1, 0.5, seed=19)
    rowptr, colidx, val = oracle.csr_from_dense(layer, w)
    off = oracle.lower_offsets(layer, rowptr, colidx)
    Hp, Wp = layer.H + 2 * layer.pad, layer.W + 2 * layer.pad
    f = lambda c, y, x: (c * Hp + y) * Wp + x
    nz = np.argwhere(w.reshape(layer.K, layer.Cg, layer.R, layer.S) != 0)
    assert len(nz) == len(off)
    for j, (k, c, r, s) in enumerate(nz):
        ca = (k // layer.Kg) * layer.Cg + c
        assert off[j] == f(ca, r, s)
        for (y, x) in [(0, 0), (layer.OH - 1, layer.OW - 1), (layer.OH // 2, 0)]:
            assert off[j] + f(0, y * layer.stride, x * layer.stride) == f(ca, y * layer.stride + r, x * layer.stride + s)
        assert off[j] + f(0, (layer.OH - 1) * layer.stride, (layer.OW - 1) * layer.stride) < layer.C * Hp * Wp
    # ascending within a row
    for k in range(layer.K):
        seg = off[rowptr[k]:rowptr[k + 1]]
        assert np.all(np.diff(seg) > 0)


@pytest.mark.parametrize("dims", TINY)
def test_hwc_offsets_name_the_same_elements_as_chw(oracle, dims):
    """The channel-innermost layout function: for every stored weight and every output position, the
    element the HWC offset reaches in the padded HWC image is the element the CHW offset reaches in the
    padded CHW image (the images hold distinct numbers, so equal values mean the same element); and a
    convolution gathered through the HWC offsets equals the oracle's result bit for bit."""
    layer = wl.small_layer(**dims)
    x, w = rand_case(layer, 1, 0.5, seed=29)
    rowptr, colidx, val = oracle.csr_from_dense(layer, w)
    off = oracle.lower_offsets(layer, rowptr, colidx)
    off_h = oracle.lower_offsets_hwc(layer, rowptr, colidx)
    Hp, Wp, C, st = layer.H + 2 * layer.pad, layer.W + 2 * layer.pad, layer.C, layer.stride
    # closed form
    nz = np.argwhere(w != 0)
    for j, (k, c, r, s) in enumerate(nz):
        assert off_h[j] == (r * Wp + s) * C + (k // layer.Kg) * layer.Cg + c
    ident = np.arange(1, C * Hp * Wp + 1, dtype=np.int64).reshape(C, Hp, Wp)
    chw, hwc = ident.ravel(), ident.transpose(1, 2, 0).ravel()
    ys, xs = np.meshgrid(np.arange(layer.OH), np.arange(layer.OW), indexing="ij")
    shift = (ys * st * Wp + xs * st).ravel()
    assert (off[:, None] + shift[None, :]).max() < C * Hp * Wp and (off_h[:, None] + shift[None, :] * C).max() < C * Hp * Wp
    assert np.array_equal(chw[off[:, None] + shift[None, :]], hwc[off_h[:, None] + shift[None, :] * C])
    # and the convolution itself, gathered from the padded HWC image in CSR order
    ref, _ = oracle.forward_f64(layer, rowptr, off, val, x)
    xp = np.zeros((C, Hp, Wp), dtype=np.float32)
    xp[:, layer.pad:layer.pad + layer.H, layer.pad:layer.pad + layer.W] = x[0]
    img = xp.transpose(1, 2, 0).ravel().astype(np.float64)
    got = np.zeros((layer.K, layer.OH * layer.OW))
    for k in range(layer.K):
        for j in range(rowptr[k], rowptr[k + 1]):
            got[k] += np.float64(val[j]) * img[off_h[j] + shift * C]
    assert np.array_equal(got.reshape(ref.shape[1:]), ref[0])


# ------------------------------------------------------------ timed fp32 variant
def test_fp32_variant_agrees_with_fp64(oracle):
    layer = wl.small_layer(C=16, H=13, W=13, K=24, R=3, S=3, stride=1, pad=1, groups=2)
    x, w = rand_case(layer, 5, 0.2, seed=23)
    out, ab, (rowptr, colidx, off, val) = oracle.sparse_conv(layer, w, x)
    o32, used = oracle.forward_f32(layer, rowptr, off, val, x, nthreads=2)
    assert used == 2
    assert np.all(np.abs(o32 - out) <= 1e-5 * ab)
    assert np.all(o32[ab == 0] == 0)


def test_planted_mistakes_are_caught(oracle):
    """The pins have teeth: a transposed kernel or a wrong pad changes the answer."""
    layer = wl.small_layer(C=2, H=6, W=6, K=2, R=3, S=3, stride=1, pad=1, groups=1)
    x, w = rand_case(layer, 1, 0.6, seed=29)
    out, ab, _ = oracle.sparse_conv(layer, w, x)
    out_t, _, _ = oracle.sparse_conv(layer, np.ascontiguousarray(w.transpose(0, 1, 3, 2)), x)
    out_f, _, _ = oracle.sparse_conv(layer, np.ascontiguousarray(w[:, :, ::-1, ::-1]), x)
    assert np.max(np.abs(out - out_t)) > 1e-3 and np.max(np.abs(out - out_f)) > 1e-3


def test_bias_relu_epilogue_equals_library_layers(oracle):
    """The epilogue oracle against torch's conv2d(bias) + relu in fp64; a bias on the wrong axis or a clamp
    before the bias would fail (bias values straddle the outputs' range)."""
    layer = wl.small_layer(C=6, H=9, W=7, K=8, R=3, S=3, stride=1, pad=1, groups=2)
    rng = np.random.default_rng(77)
    x = rng.standard_normal((3, layer.C, layer.H, layer.W)).astype(np.float32)
    w = np.where(rng.random((layer.K, layer.Cg, 3, 3)) < 0.4, rng.standard_normal((layer.K, layer.Cg, 3, 3)), 0).astype(np.float32)
    bias = (rng.standard_normal(layer.K) * 2).astype(np.float32)
    ref, ab, _ = oracle.sparse_conv(layer, w, x)
    for b, relu in ((bias, True), (bias, False), (None, True), (None, False)):
        got, scale = oracle.bias_relu(ref, ab, b, relu)
        t = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                       torch.from_numpy(b).double() if b is not None else None, 1, 1, 1, layer.groups)
        if relu:
            t = torch.relu(t)
        assert np.allclose(got, t.numpy(), rtol=0, atol=1e-12)
        assert np.all(scale >= ab) and (b is None) == bool(np.array_equal(scale, ab))
    got, _ = oracle.bias_relu(ref, ab, bias, True)
    assert (got == 0).any() and (got > 0).any()
