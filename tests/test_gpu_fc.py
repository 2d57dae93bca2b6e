"""GPU parity of the fully connected path (sparse weights x feature-major activations) through the C ABI
against the fp64 oracle: |gpu - oracle| <= 1e-5 * (sum|w*x| + |bias|) per output."""
import sys

import numpy as np
import pytest
import torch

from oracle import spmdm_oracle as so
from paper_1608_01409_amd import binding as B

pytestmark = pytest.mark.gpu
TOL = 1e-5


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def case(K, C, N, density, seed):
    rng = np.random.default_rng(seed)
    w = np.where(rng.random((K, C)) < density, rng.standard_normal((K, C)) * 0.05, 0).astype(np.float32)
    x_t = rng.standard_normal((C, N)).astype(np.float32)
    bias = (rng.standard_normal(K) * 0.5).astype(np.float32)
    return w, x_t, bias


def run(K, C, N, density, seed, bias_on, relu, plan=None, empty_rows=()):
    w, x_t, bias = case(K, C, N, density, seed)
    for k in empty_rows:
        w[k] = 0
    say(f"fc K={K} C={C} N={N} density={density} bias={bias_on} relu={relu}")
    h = B.sconv_create_csr(B.fc_layer(C, K), w.reshape(K, C, 1, 1), plan)
    xd = torch.from_numpy(x_t).cuda()
    bd = torch.from_numpy(bias).cuda() if bias_on else None
    out = torch.full((K, N), float("nan"), device="cuda")
    B.sconv_fc_forward(h, xd, bd, relu, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    ref, ab = so.spmdm(w, x_t)
    ref, scale = so.bias_relu_t(ref, ab, bias if bias_on else None, relu)
    err = np.abs(got - ref)
    bad = err > TOL * scale
    plan_used = B.sconv_fc_plan(h, N)
    assert not bad.any(), (plan_used, int(bad.sum()), float(err.max()), np.argwhere(bad)[:5])
    if not bias_on:
        assert np.all(got[scale == 0] == 0)
    return h, plan_used, got


@pytest.mark.parametrize("N", [4, 12, 64, 256, 260, 768, 1024, 2048, 2064])
def test_batch_sizes(N):
    """One chunk, ragged chunks, several chunks per wave, and batches above 1024 cut into tiles."""
    run(77, 200, N, 0.15, seed=N, bias_on=True, relu=True, empty_rows=(3, 76))


@pytest.mark.parametrize("bias_on,relu", [(False, False), (True, False), (False, True)])
def test_epilogue_variants(bias_on, relu):
    run(130, 333, 256, 0.1, seed=5, bias_on=bias_on, relu=relu, empty_rows=(0,))


def test_many_features_split_over_workgroups():
    """Few rows, many features: the channel blocks are shared by several workgroups (partial results, reduced)."""
    _, plan, _ = run(64, 3000, 256, 0.1, seed=6, bias_on=True, relu=True)
    assert plan["splits"] > 1
    _, plan, _ = run(64, 3000, 256, 0.1, seed=6, bias_on=False, relu=False)


def test_dense_and_empty_matrices():
    run(40, 64, 128, 1.0, seed=7, bias_on=True, relu=False)
    run(40, 64, 128, 0.0, seed=8, bias_on=True, relu=True)


def test_one_handle_several_batches_and_the_batch_major_entry_point():
    """Re-planning between batch sizes, and the same handle through sconv_forward (batch-major, the direct
    kernel), an independent second path on the GPU."""
    K, C = 50, 96
    w, _, bias = case(K, C, 4, 0.2, seed=9)
    h = B.sconv_create_csr(B.fc_layer(C, K), w.reshape(K, C, 1, 1))
    rng = np.random.default_rng(10)
    for N in (256, 8, 512, 256):
        x_t = rng.standard_normal((C, N)).astype(np.float32)
        out = torch.full((K, N), float("nan"), device="cuda")
        B.sconv_fc_forward(h, torch.from_numpy(x_t).cuda(), None, False, out)
        got = out.cpu().numpy().astype(np.float64)
        ref, ab = so.spmdm(w, x_t)
        assert np.all(np.abs(got - ref) <= TOL * ab), N
        x = torch.from_numpy(np.ascontiguousarray(x_t.T).reshape(N, C, 1, 1)).cuda()
        got2 = B.sconv_forward(h, x).cpu().numpy().reshape(N, K).T.astype(np.float64)
        assert np.all(np.abs(got2 - ref) <= TOL * ab), N


def test_alexnet_fc7_full_size():
    """4096 x 4096 at density 0.1, batch 256: every output against the oracle."""
    _, plan, _ = run(4096, 4096, 256, 0.1, seed=11, bias_on=True, relu=True)
    say(f"fc7 plan {plan}")


def test_batches_the_kernel_cannot_take_are_refused():
    w, _, _ = case(8, 8, 4, 0.5, seed=12)
    h = B.sconv_create_csr(B.fc_layer(8, 8), w.reshape(8, 8, 1, 1))
    x = torch.zeros((8, 6), device="cuda")
    with pytest.raises(B.SconvError) as e:
        B.sconv_fc_forward(h, x)
    assert e.value.status == B.ERR["BATCH"]


@pytest.mark.parametrize("plan,N", [
    (dict(kernel=3, waves=16, rows_w=8, t=1), 256), (dict(kernel=4, waves=16, rows_w=8, t=1), 256),
    (dict(kernel=3, waves=8, rows_w=12, t=1), 256), (dict(kernel=4, waves=8, rows_w=12, t=1), 252),
    (dict(kernel=3, waves=8, rows_w=16, t=1), 256), (dict(kernel=4, waves=4, rows_w=16, t=1), 64),
    (dict(kernel=3, waves=16, rows_w=8, cg=1), 512), (dict(kernel=4, waves=16, rows_w=8, cg=2), 1024),
    (dict(kernel=3, waves=16, rows_w=16, cg=4), 1024), (dict(kernel=3, waves=8, rows_w=8, t=1, splits=4, cb=5), 256),
])
def test_explicit_tilings_of_both_variants(plan, N):
    """Every one-chunk shape, several chunks per wave (batches of 512 and 1024 with one column group), column
    groups and channel splits, barrier and flow variant."""
    _, used, _ = run(300, 1100, N, 0.12, seed=21, bias_on=True, relu=True, plan=plan, empty_rows=(17,))
    for key, v in plan.items():
        assert used[key] == v, (key, used)
    assert used["t"] * used["cg"] == -(-N // 256), used


def test_activations_that_are_not_16_byte_aligned():
    """Aligned activations are staged a cell (four images, 16 bytes) per lane, others a float per lane; the sums
    are formed in the same order either way, so the two results agree bit for bit."""
    K, C, N = 130, 520, 256
    w, x_t, _ = case(K, C, N, 0.1, seed=22)
    h = B.sconv_create_csr(B.fc_layer(C, K), w.reshape(K, C, 1, 1))
    aligned = torch.from_numpy(x_t).cuda()
    assert aligned.data_ptr() % 16 == 0
    flat = torch.empty(C * N + 1, device="cuda")
    shifted = flat[1:].view(C, N)
    shifted.copy_(aligned)
    assert shifted.data_ptr() % 16 == 4 and shifted.is_contiguous()
    say("fc aligned / shifted activations")
    a = B.sconv_fc_forward(h, aligned).cpu().numpy()
    oflat = torch.full((K * N + 1,), float("nan"), device="cuda")
    b = B.sconv_fc_forward(h, shifted, None, False, oflat[1:].view(K, N)).cpu().numpy()
    ref, ab = so.spmdm(w, x_t)
    assert np.all(np.abs(a.astype(np.float64) - ref) <= TOL * ab)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("N", [8, 6, 3])
def test_convolution_whose_images_are_adjacent_in_the_output(oracle, N):
    """K = 1 with a single output position: consecutive images are 4 bytes apart in the output, the case in which
    the flat-stream kernel stores the four images of a cell with one instruction (full tiles only)."""
    from paper_1608_01409_amd import workloads as wl
    layer = wl.Layer("one_output", C=24, H=3, W=3, K=1, R=3, S=3, stride=1, pad=0, groups=1)
    rng = np.random.default_rng(23)
    w = np.where(rng.random((1, 24, 3, 3)) < 0.4, rng.standard_normal((1, 24, 3, 3)), 0).astype(np.float32)
    x = rng.standard_normal((N, 24, 3, 3)).astype(np.float32)
    say(f"conv K=1 1x1 output N={N}")
    h = B.sconv_create_csr(layer, w, dict(kernel=3))
    out = torch.full((N, 1, 1, 1), float("nan"), device="cuda")
    B.sconv_forward(h, torch.from_numpy(x).cuda(), out)
    got = out.cpu().numpy().astype(np.float64)
    ref, ab, _ = oracle.sparse_conv(layer, w, x)
    assert np.all(np.abs(got - ref) <= TOL * ab), (got.ravel(), ref.ravel())
