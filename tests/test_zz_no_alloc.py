"""The entry point that allocates nothing, sconv_forward_noalloc, through the C ABI against sconv_forward:
same kernels, same order of additions, so the outputs must be equal bit for bit (and with that within the
parity tolerance of the oracle, which sconv_forward is held to elsewhere).  Its scratch is one static device
array shared by every call on the GPU: the cases run two calls in a row, the second with a smaller input,
so that what the first call left in the array cannot leak into the second."""
import ctypes as C
import sys

import numpy as np
import pytest
import torch

from paper_1608_01409_amd import binding as B
from paper_1608_01409_amd import workloads as wl

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def rand_case(layer, N, density, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, layer.C, layer.H, layer.W)).astype(np.float32)
    w = (rng.standard_normal((layer.K, layer.Cg, layer.R, layer.S)) * 0.01).astype(np.float32)
    w = np.where(rng.random(w.shape) < density, w, np.float32(0)).astype(np.float32)
    return x, w


def raw_noalloc(h, xd, out):
    """The C symbol itself, no Python-side checks in between."""
    return B.lib().sconv_forward_noalloc(h.handle, C.c_void_p(xd.data_ptr()), C.c_void_p(out.data_ptr()), xd.shape[0],
                                         C.c_void_p(torch.cuda.current_stream().cuda_stream))


def both(h, layer, x):
    xd = torch.from_numpy(x).cuda()
    ref = torch.full((x.shape[0], layer.K, layer.OH, layer.OW), float("nan"), device="cuda")
    B.sconv_forward(h, xd, ref)                      # prepares the handle for this batch size, and is the reference
    got = torch.full_like(ref, float("nan"))
    return xd, ref, got


def test_channel_splits_two_calls_second_smaller(oracle):
    """conv3's shape at batch 16 and then 8: the library splits the input channels over several workgroups,
    so the partial results go through the static scratch."""
    layer = wl.LAYERS["conv3"]
    x, w = rand_case(layer, 16, 0.1, seed=91)
    w[5] = 0
    h = B.sconv_create_csr(layer, w)
    runs = []
    for n in (16, 8):
        xd, ref, got = both(h, layer, x[:n])
        plan = B.sconv_csr_info(h)["plan"]
        say(f"noalloc conv3 N={n} plan={plan}")
        assert plan["kernel"] in (3, 4) and plan["splits"] > 1, plan
        runs.append((xd, ref, got, plan))
    # both packings are resident now; the two calls in a row, the larger input first
    for xd, ref, got, plan in runs:
        assert raw_noalloc(h, xd, got) == 0
    torch.cuda.synchronize()
    for xd, ref, got, plan in runs:
        assert not torch.isnan(got).any()
        assert torch.equal(got, ref), plan
    # and against the oracle, to the parity tolerance
    xd, ref, got, _ = runs[1]
    o, ab, _ = oracle.sparse_conv(layer, w, x[:8])
    assert np.all(np.abs(got.cpu().numpy().astype(np.float64) - o) <= 1e-5 * ab)
    # once more in the other order: the handle switches between its resident packings without allocating
    for xd, ref, got, plan in reversed(runs):
        got.fill_(float("nan"))
        assert raw_noalloc(h, xd, got) == 0
        assert torch.equal(got, ref)


def test_strided_layer_phase_images_in_the_static_scratch():
    """A strided layer keeps its re-ordered input in scratch as well; two batch sizes, the second smaller."""
    layer = wl.small_layer("strided", C=3, H=35, W=35, K=16, R=7, S=7, stride=2, pad=1, groups=1)
    x, w = rand_case(layer, 12, 0.3, seed=92)
    h = B.sconv_create_csr(layer, w)
    for n in (12, 5):
        xd, ref, got = both(h, layer, x[:n])
        say(f"noalloc strided N={n} plan={B.sconv_csr_info(h)['plan']}")
        assert raw_noalloc(h, xd, got) == 0
        assert torch.equal(got, ref)


def test_refusals():
    layer = wl.small_layer("mid", C=32, H=13, W=13, K=50, R=3, S=3, stride=1, pad=1, groups=2)
    x, w = rand_case(layer, 8, 0.2, seed=93)
    h = B.sconv_create_csr(layer, w)
    xd = torch.from_numpy(x).cuda()
    out = torch.empty((8, layer.K, layer.OH, layer.OW), device="cuda")
    assert raw_noalloc(h, xd, out) == B.ERR["PLAN"]          # never run with this batch size: nothing is on the device
    B.sconv_forward(h, xd, out)
    assert raw_noalloc(h, xd, out) == 0
    assert raw_noalloc(h, xd[:4].contiguous(), out[:4]) == B.ERR["PLAN"]   # another batch size, not prepared
    hd = B.sconv_create_csr(layer, w, dict(kernel=2))
    B.sconv_forward(hd, xd, out)
    assert raw_noalloc(hd, xd, out) == B.ERR["PLAN"]         # the direct kernel is not served
    L = B.lib()
    assert L.sconv_forward_noalloc(None, None, None, 8, None) == B.ERR["NULL"]
    assert L.sconv_forward_noalloc(h.handle, None, C.c_void_p(out.data_ptr()), 8, None) == B.ERR["NULL"]
    assert L.sconv_forward_noalloc(h.handle, C.c_void_p(xd.data_ptr()), C.c_void_p(out.data_ptr()), 0, None) == B.ERR["BATCH"]
    # more scratch than the static array holds: a padded stride-2 layer at batch 96 wants 83 MB of phase images
    big = wl.small_layer("strided-padded", C=64, H=56, W=56, K=64, R=3, S=3, stride=2, pad=1, groups=1)
    x1, w1 = rand_case(big, 96, 0.1, seed=94)
    h1 = B.sconv_create_csr(big, w1)
    x1d = torch.from_numpy(x1).cuda()
    o1 = B.sconv_forward(h1, x1d)
    need = 96 * big.C * 4 * 29 * 29 * 4
    assert need > B.NOALLOC_SCRATCH_BYTES
    o2 = torch.zeros_like(o1)
    assert raw_noalloc(h1, x1d, o2) == B.ERR["CAPACITY"]
    assert raw_noalloc(h1, x1d[:24].contiguous(), o2[:24]) == B.ERR["PLAN"]   # would fit, but batch 24 was never prepared
    B.sconv_forward(h1, x1d[:24].contiguous(), o2[:24])
    o3 = torch.full_like(o2[:24], float("nan"))
    assert raw_noalloc(h1, x1d[:24].contiguous(), o3) == 0
    assert torch.equal(o3, o2[:24])
    # an unpadded strided layer needs no scratch at all: the kernel picks the phases out of the input
    conv1 = wl.LAYERS["conv1"]
    xc, wc = rand_case(conv1, 128, 0.3, seed=95)
    hc = B.sconv_create_csr(conv1, wc)
    xcd = torch.from_numpy(xc).cuda()
    oc = B.sconv_forward(hc, xcd)
    oc2 = torch.full_like(oc, float("nan"))
    assert raw_noalloc(hc, xcd, oc2) == 0
    assert torch.equal(oc2, oc)
