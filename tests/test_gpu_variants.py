"""Every tile shape the matrix-core kernels are built in, forced through the library's tuning hooks and
checked against the oracle: each implicit-GEMM shape in both reduction orders (channel-block-major needs
C % 64 == 0, tap-major runs otherwise) for forward and backward-data on ragged and strided problems, each
backward-weight shape with several split counts, and the two-launch plans (main shape for the whole rounds,
a smaller shape for the remaining rows), and the streaming kernel for short reductions on the geometries
its row bookkeeping and epilogue distinguish.  The test asserts that the forced shape is the one that ran."""
import os

import numpy as np
import pytest
import torch

from paper_1512_01274_amd import inputs as gen
from tests import util

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mxc():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_1512_01274_amd import mxc as m
    return m


def _names(family):
    from paper_1512_01274_amd import mxc as m
    return m.mxc_tile_names(family)


class forced:
    def __init__(self, var, value):
        self.var, self.value = var, value

    def __enter__(self):
        os.environ[self.var] = self.value

    def __exit__(self, *a):
        del os.environ[self.var]


# N, C, H, W, K, R, S, stride, pad: ragged row and column tiles; C = 64 runs the channel-block-major order,
# C = 72 the tap-major one
IGEMM_SHAPES = [
    (2, 64, 19, 17, 104, 3, 3, 1, 1),
    (3, 72, 13, 15, 200, 3, 3, 1, 1),
    (2, 128, 17, 17, 72, 3, 3, 2, 1),      # stride 2: backward-data runs one launch per residue class
    (2, 192, 21, 9, 264, 1, 1, 1, 0),      # 1x1
]


def _check(mxc, oracle, dims, passes, expect):
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy = gen.random_case(hash(dims) & 0xFFFF, *dims, dtype="bf16", dist="normal")
    run = util.Runner(mxc, dims, "bf16", "nhwc")
    for name in passes:
        if name == "fwd":
            got = run.fwd(x, w)
            ref, den = oracle.conv2d_fwd(x, w, st, pad), oracle.conv2d_fwd(np.abs(x), np.abs(w), st, pad)
        elif name == "bwd_data":
            got = run.bwd_data(dy, w)
            ref = oracle.conv2d_bwd_data(dy, w, x.shape, st, pad)
            den = oracle.conv2d_bwd_data(np.abs(dy), np.abs(w), x.shape, st, pad)
        else:
            got = run.bwd_weight(x, dy)
            ref = oracle.conv2d_bwd_weight(x, dy, w.shape, st, pad)
            den = oracle.conv2d_bwd_weight(np.abs(x), np.abs(dy), w.shape, st, pad)
        ran = mxc.mxc_last_variant()
        assert ran.split(":")[-1].startswith(expect), f"{name} {dims}: wanted {expect}, ran {ran}"
        assert util.metric(got, ref, den) <= util.TOL["bf16"], (name, dims, ran)
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", name != "bwd_weight")), (name, dims, ran)


@pytest.mark.parametrize("dims", IGEMM_SHAPES)
@pytest.mark.parametrize("tile", _names(0))
def test_every_igemm_tile(mxc, oracle, tile, dims):
    with forced("MXC_FORCE_VARIANT", tile):
        _check(mxc, oracle, dims, ("fwd", "bwd_data"), tile)


@pytest.mark.parametrize("dims", [(2, 64, 19, 17, 104, 3, 3, 1, 1), (3, 72, 13, 15, 200, 3, 3, 1, 1)])
@pytest.mark.parametrize("tile", _names(0))
def test_every_igemm_tile_fused_epilogue(mxc, oracle, tile, dims):
    """bias + ReLU in the forward epilogue and the ReLU-derivative mask in the backward-data epilogue of every tile
    shape (the bias travels through LDS, ReLU acts on the packed pair, masked stores take the general store path)."""
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy = gen.random_case((hash(dims) + 3) & 0xFFFF, *dims, dtype="bf16", dist="normal")
    bias = np.linspace(-2.0, 2.0, K).astype(np.float32)
    run = util.Runner(mxc, dims, "bf16", "nhwc")
    with forced("MXC_FORCE_VARIANT", tile):
        y = torch.full((N * K * run.P * run.Q,), float("nan"), dtype=torch.bfloat16, device="cuda")
        mxc.mxc_conv2d_fwd_bias_act(*dims, run.dt, run.lay, run._in(x), run._in(w), torch.from_numpy(bias).cuda(), 1, y, run._ws(mxc.MXC_FWD))
        assert mxc.mxc_last_variant().split(":")[-1].startswith(tile)
        ref, den = oracle.conv2d_fwd_bias_act(x, w, bias, True, st, pad)
        got = run._out(y, (N, K, run.P, run.Q))
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True)), (tile, dims)
        assert np.all(got >= 0)
        dx = torch.full((N * C * H * W,), float("nan"), dtype=torch.bfloat16, device="cuda")
        mxc.mxc_conv2d_bwd_data_relu(*dims, run.dt, run.lay, run._in(dy), run._in(w), run._in(x), dx, run._ws(mxc.MXC_BWD_DATA_RELU))
        assert mxc.mxc_last_variant().split(":")[-1].startswith(tile)
        ref, den = oracle.conv2d_bwd_data_relu(dy, w, x, st, pad)
        got = run._out(dx, (N, C, H, W))
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True)), (tile, dims)
        assert np.all(got[x <= 0] == 0)


@pytest.mark.parametrize("splits", [1, 3, 0])
@pytest.mark.parametrize("dims", IGEMM_SHAPES[:3])
@pytest.mark.parametrize("tile", _names(1))
def test_every_wgrad_tile(mxc, oracle, tile, dims, splits):
    with forced("MXC_FORCE_WGRAD", tile + (f"/{splits}" if splits else "")):
        _check(mxc, oracle, dims, ("bwd_weight",), tile)


PAIRS = [
    # main shape (one whole round of it: 256 tiles at one per CU, 512 at two), shape for the remaining rows, problem
    ("igemm_128x128_k64s2_w4", "igemm_64x128_k64s3_w4", (5, 64, 120, 120, 64, 3, 3, 1, 1)),
    ("igemm_256x128_k64s3_w8", "igemm_128x64_k64s2_w4", (5, 64, 120, 120, 128, 3, 3, 1, 1)),
    ("igemm_256x256_k64s2_w8", "igemm_64x256_k64s3_w8", (5, 72, 120, 120, 256, 3, 3, 1, 1)),
    ("igemm_256x256_k64s2_w8", "igemm_192x256_k64s2_w8", (5, 64, 120, 120, 200, 1, 1, 1, 0)),
]


@pytest.mark.parametrize("main,tail,dims", PAIRS)
def test_two_launch_plans(mxc, oracle, main, tail, dims):
    with forced("MXC_FORCE_VARIANT", main + "+" + tail):
        _check(mxc, oracle, dims, ("fwd",), main + "+" + tail)


# The streaming kernel (filter tile resident on chip, persistent workgroups): 1x1 and short 3x3 reductions;
# column tiles of 32 / 64 / 128 with ragged last tiles and more than one column tile; images smaller than a
# row tile (a tile spans several images), strides and padding (row positions advance with wraps), reductions
# that end inside a stage; backward-data at stride 2 writes one residue class per launch.
STREAM_SHAPES = [
    (3, 64, 29, 31, 64, 1, 1, 1, 0),
    (2, 192, 28, 28, 96, 1, 1, 1, 0),
    (5, 256, 7, 7, 40, 1, 1, 1, 0),
    (2, 64, 30, 30, 264, 1, 1, 1, 0),
    (2, 128, 27, 27, 128, 1, 1, 2, 0),
    (2, 8, 33, 35, 64, 3, 3, 1, 1),
    (2, 16, 19, 23, 32, 3, 3, 2, 1),
    (70, 24, 5, 3, 16, 3, 3, 1, 1),
    (1, 72, 57, 57, 24, 1, 1, 1, 0),
]


@pytest.mark.parametrize("dims", STREAM_SHAPES)
def test_stream_kernel(mxc, oracle, dims):
    with forced("MXC_FORCE_VARIANT", "igemm_stream"):
        _check(mxc, oracle, dims, ("fwd", "bwd_data"), "igemm_stream")


# every form the streaming kernel is built in (compute waves x ring stages), on problems whose filter tile
# fits beside the deepest ring
@pytest.mark.parametrize("form", ["4x4", "8x3", "4x3"])
@pytest.mark.parametrize("dims", [STREAM_SHAPES[i] for i in (0, 5, 6, 7, 8)])
def test_stream_kernel_forms(mxc, oracle, dims, form):
    with forced("MXC_FORCE_VARIANT", "igemm_stream"), forced("MXC_STREAM_SHAPE", form):
        _check(mxc, oracle, dims, ("fwd", "bwd_data"), "igemm_stream")


def _random_stream_shapes(count):
    """Short-reduction problems drawn at random (fixed seed): 1x1 to 3x3 filters, strides 1-2, every padding up to
    the filter size, channel counts from 8 to 136 in steps of 8, images from 1 to 40 pixels a side, batches 1-70."""
    rng = np.random.Generator(np.random.Philox(key=20240))
    out = []
    while len(out) < count:
        R, S = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        st = int(rng.integers(1, 3))
        pad = int(rng.integers(0, max(R, S)))
        H, W = int(rng.integers(1, 41)), int(rng.integers(1, 41))
        C, K = 8 * int(rng.integers(1, 18)), 8 * int(rng.integers(1, 18))
        N = int(rng.choice([1, 2, 3, 5, 70]))
        if H + 2 * pad < R or W + 2 * pad < S or N * H * W > 60000 or R * S * max(C, K) > 640:
            continue
        out.append((N, C, H, W, K, R, S, st, pad))
    return out


@pytest.mark.parametrize("dims", _random_stream_shapes(40))
def test_stream_kernel_random_shapes(mxc, oracle, dims):
    """The streaming kernel asked for on random short-reduction problems (where it declines, the tiled kernel runs:
    either way the result must match the oracle)."""
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy = gen.random_case(hash(dims) & 0xFFFF, *dims, dtype="bf16", dist="normal")
    run = util.Runner(mxc, dims, "bf16", "nhwc")
    with forced("MXC_FORCE_VARIANT", "igemm_stream"):
        got = run.fwd(x, w)
        v1 = mxc.mxc_last_variant()
        ref, den = oracle.conv2d_fwd(x, w, st, pad), oracle.conv2d_fwd(np.abs(x), np.abs(w), st, pad)
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True)), (dims, v1)
        got = run.bwd_data(dy, w)
        v2 = mxc.mxc_last_variant()
        ref = oracle.conv2d_bwd_data(dy, w, x.shape, st, pad)
        den = oracle.conv2d_bwd_data(np.abs(dy), np.abs(w), x.shape, st, pad)
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True)), (dims, v2)


def test_stream_kernel_epilogue(mxc, oracle):
    """bias + ReLU on the forward output and the ReLU-derivative mask on the backward-data output, both applied
    by the streaming kernel's epilogue."""
    dims = (3, 64, 26, 22, 96, 1, 1, 1, 0)
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy = gen.random_case(77, *dims, dtype="bf16", dist="normal")
    bias = np.linspace(-1.0, 1.0, K).astype(np.float32)
    run = util.Runner(mxc, dims, "bf16", "nhwc")
    with forced("MXC_FORCE_VARIANT", "igemm_stream"):
        y = torch.empty(N * K * H * W, dtype=torch.bfloat16, device="cuda")
        mxc.mxc_conv2d_fwd_bias_act(*dims, run.dt, run.lay, run._in(x), run._in(w), torch.from_numpy(bias).cuda(), 1, y, run._ws(mxc.MXC_FWD))
        assert mxc.mxc_last_variant().split(":")[-1] == "igemm_stream"
        ref, den = oracle.conv2d_fwd_bias_act(x, w, bias, True, st, pad)
        got = run._out(y, (N, K, H, W))
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True))
        dx = torch.empty(N * C * H * W, dtype=torch.bfloat16, device="cuda")
        mxc.mxc_conv2d_bwd_data_relu(*dims, run.dt, run.lay, run._in(dy), run._in(w), run._in(x), dx, run._ws(mxc.MXC_BWD_DATA_RELU))
        assert mxc.mxc_last_variant().split(":")[-1] == "igemm_stream"
        ref, den = oracle.conv2d_bwd_data_relu(dy, w, x, st, pad)
        got = run._out(dx, (N, C, H, W))
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True))
        assert np.all(got[x <= 0] == 0)


def test_stream_kernel_declines_long_reductions(mxc, oracle):
    """A filter tile that does not fit on chip: the forced name is ignored and a tile of the other kernel runs."""
    dims = (2, 256, 12, 12, 128, 3, 3, 1, 1)
    x, w, dy = gen.random_case(5, *dims, dtype="bf16", dist="normal")
    run = util.Runner(mxc, dims, "bf16", "nhwc")
    with forced("MXC_FORCE_VARIANT", "igemm_stream"):
        got = run.fwd(x, w)
    assert "stream" not in mxc.mxc_last_variant()
    ref, den = oracle.conv2d_fwd(x, w, 1, 1), oracle.conv2d_fwd(np.abs(x), np.abs(w), 1, 1)
    assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True))


# the window kernel (multi-tap stride-1 layers of at most 64 channels, input window and filter resident in LDS):
# filters 1x2 to 3x5, every padding up to the filter size, 16 to 64 channels, one and several column tiles, images
# narrower and wider than a patch row, ragged patches on both axes
WINDOW_SHAPES = [
    ((2, 64, 19, 17, 64, 3, 3, 1, 1), ("fwd", "bwd_data")),
    ((3, 48, 13, 40, 96, 3, 3, 1, 1), ("fwd",)),            # three k-steps, two column tiles (the second ragged)
    ((3, 96, 13, 40, 48, 3, 3, 1, 1), ("bwd_data",)),       # ... and its mirror image for backward-data
    ((2, 32, 27, 27, 32, 3, 5, 1, 1), ("fwd", "bwd_data")), # 15 taps, two k-steps, 32-column tile
    ((1, 16, 40, 36, 16, 3, 3, 1, 1), ("fwd", "bwd_data")), # one k-step
    ((2, 48, 21, 70, 64, 3, 3, 1, 0), ("fwd", "bwd_data")), # no padding: the output grid is smaller than the input
    ((2, 64, 21, 23, 48, 3, 3, 1, 2), ("fwd", "bwd_data")), # padding 2: larger
    ((1, 64, 70, 45, 16, 3, 3, 1, 1), ("fwd", "bwd_data")), # several patches per image, 16 output channels
    ((5, 64, 9, 11, 64, 3, 3, 1, 1), ("fwd", "bwd_data")),  # images smaller than a patch
    ((2, 32, 18, 18, 48, 1, 2, 1, 0), ("fwd", "bwd_data")), # two taps: the fewest the kernel takes
    ((1, 64, 1, 50, 64, 3, 3, 1, 1), ("fwd", "bwd_data")),  # one-row image
    ((16, 64, 56, 56, 64, 3, 3, 1, 1), ("fwd", "bwd_data")),  # every workgroup walks several patches
]


@pytest.mark.parametrize("dims,passes", WINDOW_SHAPES)
def test_window_kernel(mxc, oracle, dims, passes):
    with forced("MXC_FORCE_VARIANT", "igemm_window"):
        _check(mxc, oracle, dims, passes, "igemm_window")


@pytest.mark.parametrize("patch", ["8x32", "4x64", "2x64", "3x32"])
def test_window_kernel_patch_shapes(mxc, oracle, patch):
    """Patch shapes forced through the tuning hook (32 output columns: the filter tile leaves room for the wider
    windows): the result does not depend on how the output grid is cut."""
    dims = (2, 64, 30, 141, 32, 3, 3, 1, 1)
    with forced("MXC_FORCE_VARIANT", "igemm_window"), forced("MXC_WINDOW_PATCH", patch):
        _check(mxc, oracle, dims, ("fwd",), "igemm_window")


def test_window_kernel_epilogue(mxc, oracle):
    """bias + ReLU applied by the window kernel's epilogue; the masked backward-data form is not its to run."""
    dims = (3, 64, 20, 22, 64, 3, 3, 1, 1)
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy = gen.random_case(78, *dims, dtype="bf16", dist="normal")
    bias = np.linspace(-1.0, 1.0, K).astype(np.float32)
    run = util.Runner(mxc, dims, "bf16", "nhwc")
    with forced("MXC_FORCE_VARIANT", "igemm_window"):
        y = torch.empty(N * K * H * W, dtype=torch.bfloat16, device="cuda")
        mxc.mxc_conv2d_fwd_bias_act(*dims, run.dt, run.lay, run._in(x), run._in(w), torch.from_numpy(bias).cuda(), 1, y, run._ws(mxc.MXC_FWD))
        assert mxc.mxc_last_variant().split(":")[-1] == "igemm_window"
        ref, den = oracle.conv2d_fwd_bias_act(x, w, bias, True, st, pad)
        got = run._out(y, (N, K, H, W))
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True))
        dx = torch.empty(N * C * H * W, dtype=torch.bfloat16, device="cuda")
        mxc.mxc_conv2d_bwd_data_relu(*dims, run.dt, run.lay, run._in(dy), run._in(w), run._in(x), dx, run._ws(mxc.MXC_BWD_DATA_RELU))
        assert "window" not in mxc.mxc_last_variant()
        ref, den = oracle.conv2d_bwd_data_relu(dy, w, x, st, pad)
        got = run._out(dx, (N, C, H, W))
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True))


def test_window_kernel_declines(mxc, oracle):
    """1x1 filters, strided layers, more than 64 channels and channel counts that are not a multiple of 16: the
    forced name is ignored and a tile of the other kernel runs."""
    for dims in [(2, 64, 12, 12, 64, 1, 1, 1, 0), (2, 64, 12, 12, 64, 3, 3, 2, 1), (2, 40, 12, 12, 64, 3, 3, 1, 1), (2, 80, 12, 12, 64, 3, 3, 1, 1)]:
        N, C, H, W, K, R, S, st, pad = dims
        x, w, dy = gen.random_case(6, *dims, dtype="bf16", dist="normal")
        run = util.Runner(mxc, dims, "bf16", "nhwc")
        with forced("MXC_FORCE_VARIANT", "igemm_window"):
            got = run.fwd(x, w)
        assert "window" not in mxc.mxc_last_variant()
        ref, den = oracle.conv2d_fwd(x, w, st, pad), oracle.conv2d_fwd(np.abs(x), np.abs(w), st, pad)
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True)), dims


def _random_window_shapes(count):
    """Multi-tap stride-1 problems drawn at random (fixed seed): 1x2 to 3x3 filters, every padding up to the filter
    size, 16 to 64 channels in steps of 16 on the reduction side, 8 to 136 output channels, images from 1 to 90
    pixels a side, batches 1-9."""
    rng = np.random.Generator(np.random.Philox(key=20251))
    out = []
    while len(out) < count:
        R, S = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        pad = int(rng.integers(0, max(R, S)))
        H, W = int(rng.integers(1, 91)), int(rng.integers(1, 91))
        C, K = 16 * int(rng.integers(1, 5)), 8 * int(rng.integers(1, 18))
        N = int(rng.choice([1, 2, 3, 9]))
        if R * S < 2 or H + 2 * pad < R or W + 2 * pad < S or N * H * W > 40000:
            continue
        out.append((N, C, H, W, K, R, S, 1, pad))
    return out


@pytest.mark.parametrize("dims", _random_window_shapes(30))
def test_window_kernel_random_shapes(mxc, oracle, dims):
    """The window kernel asked for on random problems; forward always fits it (at most 64 input channels), backward-
    data where K is a multiple of 16 up to 64 - elsewhere the tiled kernel runs; either way the result must match
    the oracle."""
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy = gen.random_case(hash(dims) & 0xFFFF, *dims, dtype="bf16", dist="normal")
    run = util.Runner(mxc, dims, "bf16", "nhwc")
    with forced("MXC_FORCE_VARIANT", "igemm_window"):
        got = run.fwd(x, w)
        v1 = mxc.mxc_last_variant()
        assert v1.endswith("igemm_window"), (dims, v1)
        ref, den = oracle.conv2d_fwd(x, w, st, pad), oracle.conv2d_fwd(np.abs(x), np.abs(w), st, pad)
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True)), (dims, v1)
        got = run.bwd_data(dy, w)
        v2 = mxc.mxc_last_variant()
        assert v2.endswith("igemm_window") == (K % 16 == 0 and K <= 64 and C % 8 == 0), (dims, v2)
        ref = oracle.conv2d_bwd_data(dy, w, x.shape, st, pad)
        den = oracle.conv2d_bwd_data(np.abs(dy), np.abs(w), x.shape, st, pad)
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True)), (dims, v2)
