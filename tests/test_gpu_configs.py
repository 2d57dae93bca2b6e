"""GPU parity at the benchmark configurations' stated sizes: every layer of every configuration is run once
as one full-size launch, with the tiling the library chooses for that batch (the one bench.py and report.py
time), and EVERY output of EVERY image is compared with the fp64 oracle.

Tolerance as in test_gpu_parity.py: |gpu - oracle| <= 1e-5 * sum|w*x| per output; exactly zero where that
sum is zero.  The output buffer is filled with NaN first and must hold none afterwards, so an image tile, a
band or a row tile that some workgroup failed to write cannot pass."""
import sys

import numpy as np
import pytest
import torch

from paper_1608_01409_amd import binding as B
from paper_1608_01409_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 1e-5


def say(msg):
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def full_check(layer, w, x, oracle, what, plan=None):
    N = x.shape[0]
    say(f"{what} layer={layer.name} N={N} nnz={int(np.count_nonzero(w))}")
    h = B.sconv_create_csr(layer, w, plan)
    xd = torch.from_numpy(x).cuda()
    out = torch.full((N, layer.K, layer.OH, layer.OW), float("nan"), device="cuda")
    B.sconv_forward(h, xd, out)
    torch.cuda.synchronize()
    info = B.sconv_csr_info(h)
    if plan is None:
        # the tiling under test is the one the reports and the benchmark time: the cost model's first choice for N
        assert info["plan"] == B.sconv_rank_plans(h, N, 1)[0], (info["plan"], B.sconv_rank_plans(h, N, 1)[0])
    got = out.cpu().numpy()
    del out, xd
    assert not np.isnan(got).any(), (what, info["plan"], np.argwhere(np.isnan(got))[:5])
    ref, ab, _ = oracle.sparse_conv(layer, w, x)
    err = np.abs(got.astype(np.float64) - ref)
    bad = err > TOL * ab
    assert not bad.any(), (what, info["plan"], int(bad.sum()), float(err.max()), np.argwhere(bad)[:5])
    assert np.all(got[ab == 0] == 0)
    return info


def test_config1_conv3_batch1(oracle):
    (name, N, dens), = wl.CONFIGS[0]
    layer = wl.LAYERS[name]
    x, w = wl.make_case(0, 0, layer, N, dens)
    full_check(layer, w, x, oracle, "config1")
    full_check(layer, w, x, oracle, "config1-per-row-streams", dict(kernel=1, nt=1, cb=32, waves=8, cg=1, rows_w=8, t=3))
    full_check(layer, w, x, oracle, "config1-direct", dict(kernel=2))


@pytest.mark.parametrize("li", range(4))
def test_config2_alexnet_batch256_every_image(oracle, li):
    """conv2-5 at batch 256 and density 0.10 exactly as bench.py launches them; all 256 images compared."""
    name, N, dens = wl.CONFIGS[1][li]
    layer = wl.LAYERS[name]
    x, w = wl.make_case(1, li, layer, N, dens)
    full_check(layer, w, x, oracle, f"config2-{name}")


@pytest.mark.parametrize("li", range(4))
def test_config2_alexnet_batch256_every_image_flow_variant(oracle, li):
    """The same four launches through the flow variant of the kernel (three buffers, counters instead of barriers)."""
    name, N, dens = wl.CONFIGS[1][li]
    layer = wl.LAYERS[name]
    x, w = wl.make_case(1, li, layer, N, dens)
    info = full_check(layer, w, x, oracle, f"config2-flow-{name}", dict(kernel=4))
    assert info["plan"]["kernel"] == 4


@pytest.mark.parametrize("dens", wl.SWEEP_DENSITIES)
@pytest.mark.parametrize("li", range(4))
def test_config3_density_sweep_batch256_every_image(oracle, li, dens):
    """Every (layer, density) point of the sweep report.py times, same seeds, batch 256, all images."""
    name, N, _ = wl.CONFIGS[1][li]
    layer = wl.LAYERS[name]
    x, w = wl.make_case(2, li, layer, N, dens)
    full_check(layer, w, x, oracle, f"config3-{name}-x{dens}")


@pytest.mark.parametrize("cluster", ["channels", "positions"])
@pytest.mark.parametrize("li,name", [(0, "conv3"), (1, "conv4")])
def test_config4_skewed_rows_batch256_every_image(oracle, li, name, cluster):
    """Power-law row densities with 20 % empty rows at batch 256, nonzeros clustered by input channel (the
    pattern report.py times) and by kernel position inside a channel."""
    layer = wl.LAYERS[name]
    x, w = wl.make_case(3, li, layer, 256, 0.10, skewed=True, cluster=cluster)
    nnz_row = (w.reshape(layer.K, -1) != 0).sum(1)
    assert (nnz_row == 0).sum() >= 0.15 * layer.K and nnz_row.max() > 3 * nnz_row.mean()
    full_check(layer, w, x, oracle, f"config4-{name}-{cluster}")


@pytest.mark.parametrize("li", range(3))
def test_config5_googlenet_like_and_strided_batch64_every_image(oracle, li):
    name, N, dens = wl.CONFIGS[4][li]
    layer = wl.LAYERS[name]
    x, w = wl.make_case(4, li, layer, N, dens)
    full_check(layer, w, x, oracle, f"config5-{name}")


@pytest.mark.parametrize("li", range(2))
def test_one_by_one_layers_batch64_every_image(oracle, li):
    name, N, dens = wl.CONFIGS[5][li]
    layer = wl.LAYERS[name]
    x, w = wl.make_case(5, li, layer, N, dens)
    full_check(layer, w, x, oracle, f"1x1-{name}")
