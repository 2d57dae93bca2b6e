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
