"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs, element by element.

Tolerance (fp32 accumulation on the GPU against the oracle's fp64 sum):
|gpu - oracle| <= 1e-5 * sum|w*x| per output element; where that sum is zero
(no nonzero reaches a real input) the GPU value must be exactly zero."""
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


def check(layer, w, x, oracle, plan=None, images=None, what=""):
    """Run the library on all of x; compare the images listed (default: all) with the oracle."""
    say(f"{what} layer={layer} N={x.shape[0]} plan={plan}")
    h = B.sconv_create_csr(layer, w, plan)
    info = B.sconv_csr_info(h)
    xd = torch.from_numpy(x).cuda()
    # NaN first: an output the kernel fails to write must not pass on what an earlier case left there
    out = torch.full((x.shape[0], layer.K, info["OH"], info["OW"]), float("nan"), device="cuda")
    B.sconv_forward(h, xd, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    idx = np.arange(x.shape[0]) if images is None else np.asarray(images)
    ref, ab, _ = oracle.sparse_conv(layer, w, x[idx])
    err = np.abs(got[idx].astype(np.float64) - ref)
    bad = err > TOL * ab
    assert not bad.any(), (what, info["plan"], int(bad.sum()), float(err.max()), np.argwhere(bad)[:5])
    assert np.all(got[idx][ab == 0] == 0)
    return got, info


def rand_case(layer, N, density, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, layer.C, layer.H, layer.W)).astype(np.float32)
    w = (rng.standard_normal((layer.K, layer.Cg, layer.R, layer.S)) * 0.01).astype(np.float32)
    if density < 1:
        w = np.where(rng.random(w.shape) < density, w, np.float32(0)).astype(np.float32)
    return x, w


MID = wl.small_layer("mid", C=32, H=13, W=13, K=50, R=3, S=3, stride=1, pad=1, groups=2)

PLANS = [
    None,
    dict(kernel=2),
    dict(kernel=1, nt=4, cb=8, waves=8, cg=1, rows_w=6, t=3),
    dict(kernel=1, nt=4, cb=5, waves=4, cg=1, rows_w=4, t=3),
    dict(kernel=1, nt=4, cb=16, waves=16, cg=1, rows_w=8, t=3),
    dict(kernel=1, nt=8, cb=4, waves=8, cg=2, rows_w=6, t=3),
    dict(kernel=1, nt=8, cb=4, waves=8, cg=1, rows_w=3, t=6),
    dict(kernel=1, nt=8, cb=3, waves=8, cg=1, rows_w=2, t=6),
    dict(kernel=1, nt=16, cb=2, waves=16, cg=4, rows_w=6, t=3),
    dict(kernel=1, nt=1, cb=16, waves=8, cg=1, rows_w=8, t=3),
    dict(kernel=1, nt=2, cb=16, waves=4, cg=2, rows_w=8, t=3),
    dict(kernel=1, nt=4, cb=8, waves=8, cg=1, rows_w=4, t=2, band=7),   # two bands, the second ragged
    dict(kernel=1, nt=4, cb=16, waves=4, cg=1, rows_w=8, t=1, band=4),  # four bands, the last one row
    dict(kernel=1, nt=8, cb=6, waves=8, cg=2, rows_w=4, t=2, band=5),
    dict(kernel=3, nt=4, cb=8, waves=8, cg=1, rows_w=6, t=3),           # flat streams
    dict(kernel=3, nt=4, cb=5, waves=4, cg=1, rows_w=4, t=3),
    dict(kernel=3, nt=4, cb=16, waves=16, cg=1, rows_w=8, t=3),         # one block, one buffer
    dict(kernel=3, nt=4, cb=7, waves=8, cg=1, rows_w=8, t=2, band=7),
    dict(kernel=3, nt=4, cb=16, waves=16, cg=2, rows_w=16, t=1, band=7),
    dict(kernel=3, nt=4, cb=3, waves=4, cg=1, rows_w=8, t=3),
]


def flow(plan):
    """The same tiling on the flow variant of the flat-stream kernel (three buffers, counters instead of barriers)."""
    return dict(plan, kernel=4)


PLANS += [flow(p) for p in PLANS if p and p.get("kernel") == 3]


@pytest.mark.parametrize("plan", PLANS, ids=[str(i) for i in range(len(PLANS))])
def test_every_kernel_shape_on_a_ragged_batch(oracle, plan):
    # 21 images: several tiles of 4/8/16 and a ragged last one; 25 rows per group: ragged row tiles
    x, w = rand_case(MID, 21, 0.15, seed=31)
    w[7] = 0
    w[30:34] = 0
    check(MID, w, x, oracle, plan, what="ragged")


BIG = wl.small_layer("big", C=10, H=27, W=27, K=42, R=5, S=5, stride=1, pad=2, groups=2)
WIDE = wl.small_layer("wide", C=3, H=21, W=57, K=14, R=3, S=3, stride=1, pad=0, groups=1)
# every accumulator shape (T, R) of the flat-stream kernel: T follows from the band height, R = rows_w
FLAT_SHAPES = [
    (MID, dict(kernel=3, nt=4, cb=7, waves=4, cg=1, rows_w=16, t=1, band=4)),
    (MID, dict(kernel=3, nt=4, cb=7, waves=8, cg=1, rows_w=8, t=2, band=9)),
    (MID, dict(kernel=3, nt=4, cb=7, waves=4, cg=1, rows_w=12, t=2, band=9)),
    (MID, dict(kernel=3, nt=4, cb=7, waves=8, cg=1, rows_w=4, t=3)),
    (MID, dict(kernel=3, nt=4, cb=7, waves=4, cg=1, rows_w=6, t=3)),
    (MID, dict(kernel=3, nt=4, cb=7, waves=4, cg=1, rows_w=8, t=3)),
    (BIG, dict(kernel=3, nt=4, cb=2, waves=8, cg=1, rows_w=4, t=4, band=7)),
    (BIG, dict(kernel=3, nt=4, cb=2, waves=8, cg=1, rows_w=5, t=4, band=7)),
    (BIG, dict(kernel=3, nt=4, cb=2, waves=8, cg=1, rows_w=3, t=5, band=9)),
    (BIG, dict(kernel=3, nt=4, cb=2, waves=8, cg=1, rows_w=4, t=5, band=9)),
    (BIG, dict(kernel=3, nt=4, cb=2, waves=8, cg=1, rows_w=3, t=6, band=13)),
    (BIG, dict(kernel=3, nt=4, cb=2, waves=16, cg=1, rows_w=2, t=7, band=14)),
    (BIG, dict(kernel=3, nt=4, cb=3, waves=16, cg=1, rows_w=3, t=7, band=14)),
    (BIG, dict(kernel=3, nt=4, cb=2, waves=16, cg=2, rows_w=3, t=7, band=27)),
    (BIG, dict(kernel=3, nt=4, cb=1, waves=16, cg=1, rows_w=1, t=13, band=27)),
    # lanes as blocks of rows x columns (strips): 27 columns in 3 strips of 9, bands of 7 rows (the last has 6)
    (BIG, dict(kernel=3, nt=4, cb=2, waves=8, cg=1, rows_w=4, t=3, band=7, strip=9)),
    (BIG, dict(kernel=3, nt=4, cb=3, waves=8, cg=1, rows_w=6, t=3, band=7, strip=9)),
    (BIG, dict(kernel=3, nt=4, cb=2, waves=8, cg=1, rows_w=8, t=3, band=5, strip=9)),
    (BIG, dict(kernel=3, nt=4, cb=2, waves=16, cg=2, rows_w=6, t=3, band=14, strip=9)),   # two waves stacked
    (BIG, dict(kernel=3, nt=4, cb=1, waves=16, cg=4, rows_w=8, t=3, band=20, strip=9)),  # four waves stacked
    (WIDE, dict(kernel=3, nt=4, cb=2, waves=16, cg=1, rows_w=2, t=7, band=8, strip=8)),   # 55 columns in 7 strips of 8
    (WIDE, dict(kernel=3, nt=4, cb=1, waves=16, cg=2, rows_w=3, t=7, band=12, strip=8)),
    (MID, dict(kernel=3, nt=4, cb=7, waves=4, cg=1, rows_w=3, t=7, band=8, strip=8)),    # strips far wider than the image
]


FLAT_SHAPES += [(layer, flow(p)) for layer, p in FLAT_SHAPES]


def _shape_id(p):
    return (f"k{p['kernel']}T{p['t']}R{p['rows_w']}cg{p['cg']}cb{p['cb']}w{p['waves']}" +
            (f"strip{p['strip']}b{p['band']}" if p.get("strip") else ""))


@pytest.mark.parametrize("case", FLAT_SHAPES, ids=[_shape_id(p) for _, p in FLAT_SHAPES])
def test_every_flat_stream_shape(oracle, case):
    layer, plan = case
    x, w = rand_case(layer, 9, 0.2, seed=61)
    w[3] = 0                      # an empty row
    w[layer.K - 1, :, 1:, :] = 0  # a short row
    _, info = check(layer, w, x, oracle, plan, what="flat-shape")
    assert {k: info["plan"][k] for k in plan} == plan


def test_tiling_follows_the_batch_size(oracle):
    """One handle, three batch sizes: the library re-plans and re-packs between them."""
    layer = wl.small_layer("replan", C=24, H=28, W=28, K=64, R=3, S=3, stride=1, pad=1, groups=1)
    x, w = rand_case(layer, 40, 0.2, seed=63)
    h = B.sconv_create_csr(layer, w)
    plans = []
    for n in (40, 8, 40, 5, 2):
        xd = torch.from_numpy(x[:n]).cuda()
        out = torch.full((n, layer.K, layer.OH, layer.OW), float("nan"), device="cuda")
        B.sconv_forward(h, xd, out)
        got = out.cpu().numpy()
        ref, ab, _ = oracle.sparse_conv(layer, w, x[:n])
        assert np.all(np.abs(got - ref) <= TOL * ab), n
        plans.append(B.sconv_csr_info(h)["plan"])
    r, o, v = B.sconv_csr_unpack(h, 1)
    er, eo, ev = B.sconv_csr_export(h)
    assert np.array_equal(r, er) and np.array_equal(o, eo) and np.array_equal(v.view(np.uint32), ev.view(np.uint32))


def _random_layer(rng):
    groups = int(rng.choice([1, 1, 2, 3]))
    R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    stride = int(rng.choice([1, 1, 1, 2, 3]))
    pad = int(rng.integers(0, 4))
    H = int(rng.integers(max(R - 2 * pad, 1), 31)) + (0 if R - 2 * pad <= 0 else 0)
    W = int(rng.integers(max(S - 2 * pad, 1), 31))
    H, W = max(H, R - 2 * pad, 1), max(W, S - 2 * pad, 1)
    return wl.small_layer("rnd", C=groups * int(rng.integers(1, 9)), H=H, W=W, K=groups * int(rng.integers(1, 20)),
                          R=R, S=S, stride=stride, pad=pad, groups=groups)


@pytest.mark.parametrize("seed", range(40))
def test_random_layers_automatic_plan(oracle, seed):
    """Seeded random geometry (kernel sizes 1-5, strides 1-3, pads 0-3, groups 1-3, images up to 30x30),
    random density and batch: whatever the library chooses must match the oracle, and so must its choice
    among the tilings of the flow variant."""
    rng = np.random.default_rng(7000 + seed)
    layer = _random_layer(rng)
    N = int(rng.choice([4, 5, 7, 12, 17]))
    x, w = rand_case(layer, N, float(rng.choice([0.05, 0.2, 0.5, 1.0])), seed=8000 + seed)
    if layer.K > 2:
        w[int(rng.integers(0, layer.K))] = 0
    check(layer, w, x, oracle, None, what=f"random-{seed}")
    _, info = check(layer, w, x, oracle, dict(kernel=4), what=f"random-flow-{seed}")
    assert info["plan"]["kernel"] == 4


@pytest.mark.parametrize("seed", range(30))
def test_random_layers_with_many_channels_both_flat_variants(oracle, seed):
    """Up to 40 input channels per group and 70 rows, so that a workgroup walks several channel blocks, with the
    barrier or the flow variant forced, 4 to 16 waves and sometimes a channel split: the block ring, the landing
    counters, the staging by the first waves and the reduction of partial results on shapes nobody chose.
    A tiling the library refuses for the drawn layer is a skipped case, not a failure."""
    rng = np.random.default_rng(71000 + seed)
    groups = int(rng.choice([1, 1, 2]))
    R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
    stride, pad = int(rng.choice([1, 1, 1, 2, 4])), int(rng.integers(0, 3))
    H = max(int(rng.integers(1, 40)), R - 2 * pad, 1)
    W = max(int(rng.integers(1, 40)), S - 2 * pad, 1)
    layer = wl.small_layer("rnd", C=groups * int(rng.integers(1, 40)), H=H, W=W, K=groups * int(rng.integers(1, 70)),
                           R=R, S=S, stride=stride, pad=pad, groups=groups)
    N = int(rng.choice([4, 5, 8, 12, 17, 33, 64]))
    x, w = rand_case(layer, N, float(rng.choice([0.03, 0.2, 0.6, 1.0])), seed=72000 + seed)
    plan = dict(kernel=int(rng.choice([3, 4, 4])))
    if rng.random() < 0.5:
        plan["waves"] = int(rng.choice([4, 8, 16]))
    if rng.random() < 0.3:
        plan["splits"] = int(rng.choice([2, 3]))
    try:
        _, info = check(layer, w, x, oracle, plan, what=f"random-many-channels-{seed}")
    except B.SconvError as e:
        if e.status == B.ERR["PLAN"]:
            pytest.skip(f"tiling {plan} not runnable for {layer}")
        raise
    assert info["plan"]["kernel"] == plan["kernel"]


SHAPES = [
    dict(C=8, H=27, W=27, K=16, R=5, S=5, stride=1, pad=2, groups=2),
    dict(C=6, H=28, W=28, K=12, R=3, S=3, stride=1, pad=1, groups=1),
    dict(C=4, H=28, W=28, K=12, R=5, S=5, stride=1, pad=2, groups=1),
    dict(C=6, H=9, W=17, K=10, R=3, S=5, stride=1, pad=0, groups=1),
    dict(C=6, H=10, W=7, K=9, R=1, S=1, stride=1, pad=0, groups=3),
    dict(C=4, H=11, W=8, K=6, R=2, S=3, stride=1, pad=3, groups=1),
    dict(C=3, H=35, W=35, K=8, R=11, S=11, stride=4, pad=0, groups=1),
    dict(C=4, H=14, W=15, K=6, R=3, S=3, stride=2, pad=1, groups=2),
    dict(C=2, H=12, W=10, K=4, R=3, S=3, stride=3, pad=2, groups=1),
]


@pytest.mark.parametrize("dims", SHAPES, ids=[str(i) for i in range(len(SHAPES))])
@pytest.mark.parametrize("N", [1, 6])
def test_layer_shapes_automatic_plan(oracle, dims, N):
    layer = wl.small_layer("shape", **dims)
    x, w = rand_case(layer, N, 0.3, seed=41 + N)
    check(layer, w, x, oracle, None, what="shape")


def test_density_one_and_zero(oracle):
    x, w = rand_case(MID, 9, 1.0, seed=43)
    check(MID, w, x, oracle, None, what="dense")
    check(MID, w, x, oracle, dict(kernel=2), what="dense-direct")
    z = np.zeros_like(w)
    for plan in (None, dict(kernel=2)):
        got, _ = check(MID, z, x, oracle, plan, what="all-zero")
        assert np.all(got == 0)


def test_linear_in_weights_on_gpu(oracle):
    x, w1 = rand_case(MID, 8, 0.2, seed=45)
    _, w2 = rand_case(MID, 8, 0.2, seed=46)
    w1 = (np.round(w1 * 2 ** 16) / 2 ** 16).astype(np.float32)
    w2 = (np.round(w2 * 2 ** 16) / 2 ** 16).astype(np.float32)
    g1, _ = check(MID, w1, x, oracle, None, what="lin-1")
    g2, _ = check(MID, w2, x, oracle, None, what="lin-2")
    g12, _ = check(MID, (0.5 * w1 - 2 * w2).astype(np.float32), x, oracle, None, what="lin-12")
    _, a1, _ = oracle.sparse_conv(MID, w1, x)
    _, a2, _ = oracle.sparse_conv(MID, w2, x)
    assert np.all(np.abs(g12 - (0.5 * g1.astype(np.float64) - 2 * g2)) <= 3 * TOL * (0.5 * a1 + 2 * a2))


def test_run_to_run_bit_identical_and_output_overwritten(oracle):
    x, w = rand_case(MID, 12, 0.15, seed=47)
    h = B.sconv_create_csr(MID, w)
    xd = torch.from_numpy(x).cuda()
    out = torch.full((12, MID.K, MID.OH, MID.OW), float("nan"), device="cuda")
    B.sconv_forward(h, xd, out)
    a = out.clone()
    out.fill_(123.0)
    B.sconv_forward(h, xd, out)
    torch.cuda.synchronize()
    assert torch.equal(a, out) and not torch.isnan(out).any()


def test_non_finite_inputs_stay_where_the_oracle_puts_them(oracle):
    """Padding entries of the nonzero stream multiply zeros, never the input."""
    x, w = rand_case(MID, 8, 0.15, seed=49)
    x[:, :, 0, 0] = np.inf
    x[3, 5, 6, 6] = np.nan
    h = B.sconv_create_csr(MID, w)
    got = B.sconv_forward(h, torch.from_numpy(x).cuda()).cpu().numpy()
    ref, ab, _ = oracle.sparse_conv(MID, w, x)
    fin = np.isfinite(ref)
    assert np.array_equal(np.isfinite(got), fin)
    assert np.all(np.abs(got[fin] - ref[fin]) <= TOL * ab[fin])


def test_stream_argument_is_honoured(oracle):
    x, w = rand_case(MID, 8, 0.15, seed=51)
    h = B.sconv_create_csr(MID, w)
    xd = torch.from_numpy(x).cuda()
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        out = B.sconv_forward(h, xd)
    s.synchronize()
    ref, ab, _ = oracle.sparse_conv(MID, w, x)
    assert np.all(np.abs(out.cpu().numpy() - ref) <= TOL * ab)


def check_fused(layer, w, x, oracle, plan, bias, relu, what=""):
    say(f"{what} layer={layer} N={x.shape[0]} plan={plan} bias={bias is not None} relu={relu}")
    h = B.sconv_create_csr(layer, w, plan)
    info = B.sconv_csr_info(h)
    xd = torch.from_numpy(x).cuda()
    bd = torch.from_numpy(bias).cuda() if bias is not None else None
    out = torch.full((x.shape[0], layer.K, info["OH"], info["OW"]), float("nan"), device="cuda")
    B.sconv_forward_fused(h, xd, bd, relu, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    ref, ab, _ = oracle.sparse_conv(layer, w, x)
    ref, scale = oracle.bias_relu(ref, ab, bias, relu)
    err = np.abs(got - ref)
    bad = err > TOL * scale
    assert not bad.any(), (what, info["plan"], int(bad.sum()), float(err.max()), np.argwhere(bad)[:5])
    if relu:
        assert (got >= 0).all()
    return info


EPILOGUE_PLANS = [
    None,
    dict(kernel=2),                                                      # direct kernel: a pass of its own
    dict(kernel=1, nt=4, cb=8, waves=8, cg=1, rows_w=6, t=3),            # per-row streams: a pass of its own
    dict(kernel=3, nt=4, cb=8, waves=8, cg=1, rows_w=6, t=3),            # fused
    dict(kernel=3, nt=4, cb=7, waves=4, cg=1, rows_w=16, t=1, band=4),   # 16 rows per wave
    dict(kernel=3, nt=4, cb=7, waves=4, cg=1, rows_w=12, t=2, band=9),
    dict(kernel=3, nt=4, cb=4, waves=8, cg=1, rows_w=4, t=3, splits=2),  # two workgroups share the channels (partial results + reduction)
    dict(kernel=3, nt=4, cb=3, waves=8, cg=1, rows_w=8, t=3, splits=3),  # 6 blocks in three parts
    dict(kernel=3, nt=4, cb=3, waves=8, cg=1, rows_w=8, t=3, splits=6),  # one block each
]
EPILOGUE_PLANS += [flow(p) for p in EPILOGUE_PLANS if p and p.get("kernel") == 3]


@pytest.mark.parametrize("plan", EPILOGUE_PLANS, ids=[str(i) for i in range(len(EPILOGUE_PLANS))])
def test_bias_and_relu_epilogue(oracle, plan):
    x, w = rand_case(MID, 10, 0.2, seed=71)
    w[5] = 0   # a row with no nonzeros: its outputs are max(bias, 0)
    rng = np.random.default_rng(72)
    bias = (rng.standard_normal(MID.K) * 0.05).astype(np.float32)
    for b, relu in ((bias, True), (bias, False), (None, True)):
        info = check_fused(MID, w, x, oracle, plan, b, relu, what="epilogue")
        if plan:
            assert {k: info["plan"][k] for k in plan} == plan


@pytest.mark.parametrize("kernel", [3, 4])
@pytest.mark.parametrize("splits", [2, 5])
def test_channel_splits_without_epilogue(oracle, splits, kernel):
    """Partial sums of several workgroups added up by a second launch: the plain entry point, a strip layout, a ragged batch."""
    plan = dict(kernel=kernel, nt=4, cb=1, waves=8, cg=1, rows_w=4, t=3, band=7, strip=9, splits=splits)
    x, w = rand_case(BIG, 6, 0.2, seed=73)
    _, info = check(BIG, w, x, oracle, plan, what="splits")
    assert info["plan"]["splits"] == splits


STRIDED = wl.small_layer("strided", C=8, H=23, W=21, K=12, R=5, S=3, stride=2, pad=0, groups=2)
STRIDED_PLANS = [
    dict(nt=4, cb=2, waves=4, cg=1, rows_w=8, t=2),             # two blocks per phase
    dict(nt=4, cb=4, waves=4, cg=1, rows_w=8, t=2),             # one block per phase
    dict(nt=4, cb=1, waves=8, cg=1, rows_w=8, t=2),             # four blocks per phase
    dict(nt=4, cb=3, waves=4, cg=1, rows_w=8, t=2),             # blocks straddle phases: the phase-image pass runs instead
    dict(nt=4, cb=2, waves=4, cg=1, rows_w=8, t=2, splits=2),   # channel parts that start in the middle of the phases
    dict(nt=4, cb=1, waves=4, cg=1, rows_w=12, t=2, splits=3),
    dict(nt=4, cb=2, waves=4, cg=1, rows_w=16, t=1, band=4),    # bands of output rows
]


@pytest.mark.parametrize("kernel", [3, 4])
@pytest.mark.parametrize("plan", STRIDED_PLANS, ids=[str(i) for i in range(len(STRIDED_PLANS))])
def test_strided_unpadded_layer_staged_from_the_input(oracle, plan, kernel):
    """A strided layer without padding needs no phase-image pass: the kernel picks the phases out of the
    caller's tensor while staging, provided no channel block straddles two phases.  Two groups, 5 x 3 filter,
    stride 2; ragged batch; one row without nonzeros."""
    x, w = rand_case(STRIDED, 9, 0.3, seed=83)
    w[4] = 0
    _, info = check(STRIDED, w, x, oracle, dict(plan, kernel=kernel), what="strided-direct")
    assert info["plan"]["cb"] == plan["cb"] and info["plan"]["kernel"] == kernel


def test_strided_unpadded_layer_inputs_with_non_finite_values(oracle):
    """Cells of a phase image that lie beyond the input are filled with whatever follows in memory; they must
    reach no real output, whatever they hold: here the neighbouring channels and images hold Inf and NaN."""
    layer = wl.small_layer("strided2", C=3, H=19, W=19, K=8, R=7, S=7, stride=4, pad=0, groups=1)
    x, w = rand_case(layer, 6, 0.4, seed=85)
    x[:, :, 0, 0] = np.inf
    x[:, 1, -1, -1] = np.nan
    h = B.sconv_create_csr(layer, w)
    got = B.sconv_forward(h, torch.from_numpy(x).cuda()).cpu().numpy()
    ref, ab, _ = oracle.sparse_conv(layer, w, x)
    fin = np.isfinite(ref)
    assert np.array_equal(np.isfinite(got), fin)
    assert np.all(np.abs(got[fin] - ref[fin]) <= TOL * ab[fin])
