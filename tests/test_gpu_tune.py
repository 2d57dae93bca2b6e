"""The measured choice of the tiling (sconv_tune, sconv_fc_tune) through the C ABI: whatever tiling wins,
the results stay within the parity bound of the oracle, the choice is kept per batch size, and handles
with a tiling of the caller's are refused."""
import sys

import numpy as np
import pytest
import torch

from oracle import spmdm_oracle as so
from paper_1608_01409_amd import binding as B
from paper_1608_01409_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 1e-5


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def conv_case(layer, N, density, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, layer.C, layer.H, layer.W)).astype(np.float32)
    w = (rng.standard_normal((layer.K, layer.Cg, layer.R, layer.S)) * 0.01).astype(np.float32)
    w = np.where(rng.random(w.shape) < density, w, np.float32(0)).astype(np.float32)
    return x, w


def within_bound(got, ref, ab):
    err = np.abs(got.astype(np.float64) - ref)
    return not (err > TOL * ab).any() and np.all(got[ab == 0] == 0)


LAYERS = [
    wl.small_layer("t13", C=32, H=13, W=13, K=50, R=3, S=3, stride=1, pad=1, groups=2),
    wl.small_layer("t27", C=10, H=27, W=27, K=42, R=5, S=5, stride=1, pad=2, groups=2),
    wl.small_layer("tstr", C=3, H=35, W=35, K=20, R=7, S=7, stride=2, pad=0, groups=1),
]


@pytest.mark.parametrize("layer", LAYERS, ids=[l.name for l in LAYERS])
@pytest.mark.parametrize("N", [1, 9, 40])
def test_tuned_convolution_matches_the_oracle(oracle, layer, N):
    x, w = conv_case(layer, N, 0.2, seed=100 + N)
    w[3] = 0
    say(f"tune layer={layer} N={N}")
    h = B.sconv_create_csr(layer, w)
    xd = torch.from_numpy(x).cuda()
    info = B.sconv_csr_info(h)
    ref, ab, _ = oracle.sparse_conv(layer, w, x)
    out = torch.full((N, layer.K, info["OH"], info["OW"]), float("nan"), device="cuda")
    B.sconv_tune(h, xd, out, max_plans=6)
    torch.cuda.synchronize()
    assert within_bound(out.cpu().numpy(), ref, ab), B.sconv_csr_info(h)["plan"]
    tuned = B.sconv_csr_info(h)["plan"]
    # later calls with this batch size use the tuned tiling, also through the fused entry point
    out.fill_(float("nan"))
    B.sconv_forward(h, xd, out)
    assert within_bound(out.cpu().numpy(), ref, ab)
    assert B.sconv_csr_info(h)["plan"] == tuned
    bias = torch.zeros(layer.K, device="cuda")
    out.fill_(float("nan"))
    B.sconv_forward_fused(h, xd, bias, False, out)
    assert within_bound(out.cpu().numpy(), ref, ab)
    assert B.sconv_csr_info(h)["plan"] == tuned


def test_the_choice_is_kept_per_batch_size(oracle):
    layer = LAYERS[0]
    x, w = conv_case(layer, 48, 0.15, seed=7)
    h = B.sconv_create_csr(layer, w)
    xd = torch.from_numpy(x).cuda()
    say("tune per batch size")
    B.sconv_tune(h, xd, max_plans=5)
    plan48 = B.sconv_csr_info(h)["plan"]
    B.sconv_tune(h, xd[:8].contiguous(), max_plans=5)
    plan8 = B.sconv_csr_info(h)["plan"]
    for n, plan in ((48, plan48), (8, plan8), (48, plan48)):
        got = B.sconv_forward(h, xd[:n].contiguous()).cpu().numpy()
        assert B.sconv_csr_info(h)["plan"] == plan, n
        ref, ab, _ = oracle.sparse_conv(layer, w, x[:n])
        assert within_bound(got, ref, ab), n


def test_more_candidates_than_the_search_has_and_odd_counts(oracle):
    layer = wl.small_layer("tiny", C=4, H=6, W=6, K=5, R=3, S=3, stride=1, pad=1, groups=1)
    x, w = conv_case(layer, 5, 0.5, seed=3)
    ref, ab, _ = oracle.sparse_conv(layer, w, x)
    xd = torch.from_numpy(x).cuda()
    for k in (32, 1000, 0, -3, 1):
        say(f"tune tiny max_plans={k}")
        h = B.sconv_create_csr(layer, w)
        got = B.sconv_tune(h, xd, max_plans=k).cpu().numpy()
        assert within_bound(got, ref, ab), k


def test_handles_with_a_tiling_of_the_callers_are_refused():
    layer = LAYERS[0]
    x, w = conv_case(layer, 8, 0.2, seed=4)
    xd = torch.from_numpy(x).cuda()
    for plan in (dict(kernel=3, nt=4, cb=8, waves=8, cg=1, rows_w=6, t=3), dict(kernel=3, waves=8), dict(kernel=2)):
        h = B.sconv_create_csr(layer, w, plan)
        with pytest.raises(B.SconvError) as e:
            B.sconv_tune(h, xd)
        assert e.value.status == B.ERR["PLAN"]
        B.sconv_forward(h, xd)   # the handle still works


@pytest.mark.parametrize("K,C,N", [(130, 333, 256), (64, 3000, 64), (77, 200, 2048)])
def test_tuned_fully_connected_layer_matches_the_oracle(K, C, N):
    rng = np.random.default_rng(K + N)
    w = np.where(rng.random((K, C)) < 0.1, rng.standard_normal((K, C)) * 0.05, 0).astype(np.float32)
    w[K - 1] = 0
    x_t = rng.standard_normal((C, N)).astype(np.float32)
    bias = (rng.standard_normal(K) * 0.5).astype(np.float32)
    say(f"fc tune K={K} C={C} N={N}")
    h = B.sconv_create_csr(B.fc_layer(C, K), w.reshape(K, C, 1, 1))
    xd = torch.from_numpy(x_t).cuda()
    out = torch.full((K, N), float("nan"), device="cuda")
    B.sconv_fc_tune(h, xd, out, max_plans=6)
    ref, ab = so.spmdm(w, x_t)
    assert not (np.abs(out.cpu().numpy().astype(np.float64) - ref) > TOL * ab).any()
    tuned = B.sconv_fc_plan(h, N)
    # with bias and ReLU, and after another batch size has been through the handle
    B.sconv_fc_forward(h, xd[:, :8].contiguous())
    out.fill_(float("nan"))
    B.sconv_fc_forward(h, xd, torch.from_numpy(bias).cuda(), True, out)
    assert B.sconv_fc_plan(h, N) == tuned
    ref2, scale = so.bias_relu_t(ref, ab, bias, True)
    assert not (np.abs(out.cpu().numpy().astype(np.float64) - ref2) > TOL * scale).any()


def test_fc_tune_refuses_what_fc_forward_refuses():
    layer = LAYERS[0]
    _, w = conv_case(layer, 4, 0.2, seed=5)
    h = B.sconv_create_csr(layer, w)
    lib = B.lib()
    import ctypes as C
    buf = torch.zeros(4096, device="cuda")
    p = C.c_void_p(buf.data_ptr())
    assert lib.sconv_fc_tune(h.handle, p, p, 8, 4, None) == B.ERR["DESC"]
    hf = B.sconv_create_csr(B.fc_layer(16, 8), np.ones((8, 16, 1, 1), np.float32))
    assert lib.sconv_fc_tune(hf.handle, p, p, 6, 4, None) == B.ERR["BATCH"]
    assert lib.sconv_fc_tune(hf.handle, None, p, 8, 4, None) == B.ERR["NULL"]
    assert lib.sconv_tune(None, p, p, 8, 4, None) == B.ERR["NULL"]
    assert lib.sconv_tune(h.handle, p, p, 0, 4, None) == B.ERR["BATCH"]
