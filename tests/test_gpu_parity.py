"""GPU parity: every entry point of the C ABI against the CPU oracle, element by element,
on the same seeded inputs.  Metric and tolerances: max |gpu - oracle| / D with
D = sum |a||b| over that output's taps; <= 1e-5 (fp32), <= 1e-2 (bf16); plus a much
tighter per-element bound derived from the arithmetic (fp32 accumulation + one bf16
rounding of the result), so that a dropped or misplaced tap cannot hide inside the
loose budget.  Where D == 0 (no tap reaches the element) the result must be exactly 0.
"""
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


def check_all_passes(mxc, oracle, dims, dtype, layout, x, w, dy, passes=("fwd", "bwd_data", "bwd_weight")):
    N, C, H, W, K, R, S, st, pad = dims
    run = util.Runner(mxc, dims, dtype, layout)
    ax, aw, ady = np.abs(x), np.abs(w), np.abs(dy)
    out_bf16 = dtype == "bf16"
    report = {}
    if "fwd" in passes:
        ref, den = oracle.conv2d_fwd(x, w, st, pad), oracle.conv2d_fwd(ax, aw, st, pad)
        got = run.fwd(x, w)
        report["fwd"] = (got, ref, den, out_bf16)
    if "bwd_data" in passes:
        ref, den = oracle.conv2d_bwd_data(dy, w, x.shape, st, pad), oracle.conv2d_bwd_data(ady, aw, x.shape, st, pad)
        got = run.bwd_data(dy, w)
        report["bwd_data"] = (got, ref, den, out_bf16)
    if "bwd_weight" in passes:
        ref, den = oracle.conv2d_bwd_weight(x, dy, w.shape, st, pad), oracle.conv2d_bwd_weight(ax, ady, w.shape, st, pad)
        got = run.bwd_weight(x, dy)
        report["bwd_weight"] = (got, ref, den, False)
    for name, (got, ref, den, ob) in report.items():
        assert got.shape == ref.shape, name
        err = util.metric(got, ref, den)
        assert err <= util.TOL[dtype], f"{name} {dims} {dtype} {layout}: err {err:.3e} variant {mxc.mxc_last_variant()}"
        excess = np.abs(got - ref) - util.tight_bound(ref, den, dtype, ob)
        worst = np.unravel_index(np.argmax(excess), excess.shape)
        assert excess.max() <= 0, (f"{name} {dims} {dtype} {layout}: tight bound exceeded at {worst}: "
                                   f"gpu {got[worst]!r} oracle {ref[worst]!r} D {den[worst]!r}")


# ---- config 1 (fp32 single layer), in full, both layouts -----------------------

@pytest.mark.parametrize("layout", ["nchw", "nhwc"])
def test_config1_full(mxc, oracle, layout):
    cfg = gen.CONFIGS[0]
    L, t = gen.layer_inputs(cfg, 0)
    check_all_passes(mxc, oracle, L.dims(), "f32", layout, t["x"], t["w"], t["dy"])


# ---- shape sweep: ragged tiles, strides, pads, floor remainders ----------------

SWEEP = [
    # N, C, H, W, K, R, S, stride, pad
    (1, 1, 1, 1, 1, 1, 1, 1, 0),        # smallest problem
    (2, 3, 9, 7, 5, 3, 3, 1, 1),        # H != W, odd C and K
    (1, 8, 12, 12, 16, 3, 3, 2, 1),
    (3, 16, 10, 11, 24, 1, 1, 1, 0),    # 1x1
    (2, 24, 9, 9, 40, 1, 1, 2, 0),      # 1x1 stride 2: three quarters of dx is zero fill
    (2, 5, 13, 13, 7, 5, 5, 1, 2),
    (1, 3, 35, 35, 8, 11, 11, 4, 2),    # first-layer style, (H+2pad-R) % stride != 0
    (2, 40, 7, 7, 72, 3, 3, 1, 1),      # small spatial, several channel chunks
    (1, 16, 8, 8, 16, 3, 3, 3, 0),      # stride 3, remainder rows never read
    (1, 4, 6, 6, 4, 2, 2, 1, 1),        # even filter
    (2, 8, 5, 5, 8, 3, 3, 1, 2),        # pad == R-1
    (1, 8, 4, 4, 8, 1, 1, 1, 1),        # pad > R-1 (1x1 with padding)
    (1, 136, 6, 5, 264, 3, 3, 1, 1),    # C, K beyond one tile with ragged tails
    (5, 32, 17, 17, 48, 3, 3, 2, 0),
    (1, 8, 40, 3, 8, 3, 3, 1, 1),       # tall and narrow
    (2, 3, 13, 11, 16, 3, 3, 1, 1),     # small-C paths: stride 1, W not a multiple of the column group
    (1, 2, 12, 15, 8, 5, 5, 2, 2),      # small-C, stride 2
    (2, 4, 9, 9, 8, 3, 3, 1, 0),        # C == 4, no padding
    (1, 3, 20, 20, 16, 7, 7, 2, 3),
    (1, 12, 9, 9, 16, 3, 3, 1, 1),      # C % 8 != 0, C > 4: channel-padded path
    (2, 20, 7, 8, 24, 3, 3, 2, 1),
    (1, 3, 22, 24, 8, 11, 11, 4, 2),    # space-to-depth with 4-byte aligned rows (dword copy path)
    (2, 4, 18, 21, 8, 5, 5, 2, 1),
    (2, 3, 17, 16, 8, 7, 7, 2, 3),      # strided small-C with rows of whole 16-byte chunks: four column classes
    (1, 4, 10, 12, 8, 3, 3, 2, 0),      # ... one class
    (2, 1, 9, 16, 8, 5, 5, 4, 2),       # ... C == 1, stride 4: two classes
    (1, 2, 8, 8, 16, 3, 3, 2, 1),       # ... C == 2
    (2, 16, 9, 9, 64, 3, 3, 2, 1),      # K % 64 == 0: backward-data reads the filter in place (transposed tiles), stride 2
    (1, 24, 7, 7, 128, 1, 1, 1, 0),     # ... 1x1
    (2, 8, 10, 10, 64, 5, 5, 1, 2),     # ... 5x5
    (1, 40, 8, 9, 192, 3, 3, 3, 0),     # ... stride 3, ragged output columns
    (1, 264, 6, 6, 320, 3, 3, 1, 1),    # ... several column tiles, ragged
    (2, 64, 9, 10, 64, 3, 3, 1, 1),     # C % 64 == 0: channel-block-major reduction order, one block
    (1, 128, 8, 8, 64, 3, 3, 2, 1),     # ... two blocks, stride 2 (backward-data classes with 1, 2 and 4 taps)
    (2, 192, 6, 6, 32, 5, 5, 1, 2),     # ... three blocks, 25 taps
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
@pytest.mark.parametrize("dims", SWEEP)
def test_sweep(mxc, oracle, dims, dtype, layout):
    x, w, dy = gen.random_case(hash(dims) & 0xFFFF, *dims, dtype=dtype, dist="uniform")
    check_all_passes(mxc, oracle, dims, dtype, layout, x, w, dy)


# ---- the bf16 networks at reduced batch: every layer, full tensors --------------

@pytest.mark.parametrize("cfg_idx", [1, 2, 3, 4])
def test_network_layers_reduced_batch(mxc, oracle, cfg_idx):
    cfg = gen.CONFIGS[cfg_idx]
    for li in range(len(cfg.layers)):
        L, t = gen.layer_inputs(cfg, li, batch=2)
        big = L.H >= 112
        if big:  # keep the oracle's full pass to seconds: one image for the 224/112 layers
            L, t = gen.layer_inputs(cfg, li, batch=1)
        check_all_passes(mxc, oracle, L.dims(), cfg.dtype, "nhwc", t["x"], t["w"], t["dy"])


# ---- determinism: bitwise equal results from run to run ------------------------

@pytest.mark.parametrize("dims,dtype", [((4, 32, 14, 14, 64, 3, 3, 1, 1), "bf16"), ((2, 16, 16, 16, 32, 3, 3, 1, 1), "f32"),
                                        ((3, 24, 9, 9, 40, 1, 1, 2, 0), "bf16")])
def test_bitwise_determinism(mxc, dims, dtype):
    x, w, dy = gen.random_case(5, *dims, dtype=dtype, dist="normal")
    run = util.Runner(mxc, dims, dtype, "nhwc")
    for fn, args in ((run.fwd, (x, w)), (run.bwd_data, (dy, w)), (run.bwd_weight, (x, dy))):
        a = fn(*args, return_tensor=True)
        b = fn(*args, return_tensor=True)
        av = a.view(torch.int16) if a.dtype == torch.bfloat16 else a.view(torch.int32)
        bv = b.view(torch.int16) if b.dtype == torch.bfloat16 else b.view(torch.int32)
        assert torch.equal(av, bv)


# ---- nothing outside the output is written --------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_canaries_around_outputs(mxc, dtype):
    dims = (2, 24, 9, 10, 40, 3, 3, 2, 1)
    N, C, H, W, K, R, S, st, pad = dims
    P, Q = (H + 2 * pad - R) // st + 1, (W + 2 * pad - S) // st + 1
    x, w, dy = gen.random_case(6, *dims, dtype=dtype, dist="uniform")
    dt = mxc.MXC_BF16 if dtype == "bf16" else mxc.MXC_F32
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    dx_, dw_, ddy_ = (util.to_device(util.nchw_to_nhwc(a), dtype) for a in (x, w, dy))
    GUARD = 1024
    for op, fn, a, b, n_out, odt in (
            (mxc.MXC_FWD, mxc.mxc_conv2d_fwd, dx_, dw_, N * K * P * Q, td),
            (mxc.MXC_BWD_DATA, mxc.mxc_conv2d_bwd_data, ddy_, dw_, N * C * H * W, td),
            (mxc.MXC_BWD_WEIGHT, mxc.mxc_conv2d_bwd_weight, dx_, ddy_, K * C * R * S, torch.float32)):
        n_pad = (n_out + 7) // 8 * 8          # keeps the output view 16-byte aligned
        buf = torch.full((GUARD + n_pad + GUARD,), 7.0, dtype=odt, device="cuda")
        out = buf[GUARD:GUARD + n_out]
        ws = mxc.alloc_workspace(mxc.mxc_conv2d_workspace_bytes(op, *dims, dt, mxc.MXC_NHWC))
        fn(*dims, dt, mxc.MXC_NHWC, a, b, out, ws)
        torch.cuda.synchronize()
        assert (buf[:GUARD] == 7.0).all() and (buf[GUARD + n_out:] == 7.0).all()


# ---- layout conversion: exact permutation, both directions, both element sizes --

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(1, 1, 1, 1), (2, 3, 5, 7), (3, 64, 8, 8), (2, 65, 9, 15), (1, 200, 3, 3), (2, 16, 70, 66),
                                   (2, 3, 8, 24), (3, 4, 4, 6), (1, 2, 16, 3), (2, 3, 224, 224),
                                   # rows and columns multiples of 8: the 16-byte-vector transposes, whole and ragged tiles
                                   (2, 72, 12, 10), (1, 200, 4, 6), (3, 128, 16, 16), (2, 64, 56, 56), (1, 136, 9, 8),
                                   (5, 2048, 1, 3), (1, 12, 28, 28)])
def test_layout_convert(mxc, shape, dtype):
    n, c, h, w = shape
    g = np.random.Generator(np.random.Philox(key=3))
    a = g.standard_normal(shape).astype(np.float32)
    if dtype == "bf16":
        a = gen.round_to_bf16(a)
    dt = mxc.MXC_BF16 if dtype == "bf16" else mxc.MXC_F32
    src = util.to_device(a, dtype)
    dst = torch.empty_like(src)
    mxc.mxc_layout_convert(n, c, h, w, dt, mxc.MXC_NCHW, mxc.MXC_NHWC, src, dst)
    np.testing.assert_array_equal(util.to_host_f64(dst).reshape(n, h, w, c), util.nchw_to_nhwc(a).astype(np.float64))
    back = torch.empty_like(src)
    mxc.mxc_layout_convert(n, c, h, w, dt, mxc.MXC_NHWC, mxc.MXC_NCHW, dst, back)
    np.testing.assert_array_equal(util.to_host_f64(back).reshape(shape), a.astype(np.float64))
    same = torch.empty_like(src)
    mxc.mxc_layout_convert(n, c, h, w, dt, mxc.MXC_NCHW, mxc.MXC_NCHW, src, same)
    assert torch.equal(same.view(torch.uint8), src.view(torch.uint8))


# ---- error paths on a live GPU: bad arguments launch nothing --------------------

def test_error_codes_on_gpu(mxc):
    dims = (2, 8, 6, 6, 8, 3, 3, 1, 1)
    x = torch.zeros(2 * 8 * 6 * 6, device="cuda")
    w = torch.zeros(8 * 8 * 3 * 3, device="cuda")
    y = torch.full((2 * 8 * 6 * 6,), 5.0, device="cuda")
    need = mxc.mxc_conv2d_workspace_bytes(mxc.MXC_FWD, *dims, mxc.MXC_F32, mxc.MXC_NCHW)
    assert need > 0
    with pytest.raises(mxc.MxcError) as e:
        mxc.mxc_conv2d_fwd(*dims, mxc.MXC_F32, mxc.MXC_NCHW, x, w, y, None)
    assert e.value.status == mxc.MXC_ERR_WORKSPACE
    small = mxc.alloc_workspace(need - 256)
    with pytest.raises(mxc.MxcError) as e:
        mxc.mxc_conv2d_fwd(*dims, mxc.MXC_F32, mxc.MXC_NCHW, x, w, y, small)
    assert e.value.status == mxc.MXC_ERR_WORKSPACE
    with pytest.raises(mxc.MxcError) as e:
        mxc.mxc_conv2d_fwd(*dims, mxc.MXC_F32, mxc.MXC_NHWC, x[1:], w, y, None)
    assert e.value.status == mxc.MXC_ERR_ALIGN
    with pytest.raises(mxc.MxcError) as e:
        mxc.mxc_conv2d_fwd(2, 8, 6, 6, 8, 9, 9, 1, 1, mxc.MXC_F32, mxc.MXC_NHWC, x, w, y, None)
    assert e.value.status == mxc.MXC_ERR_SHAPE
    torch.cuda.synchronize()
    assert (y == 5.0).all()


# ---- the measurement aid ----------------------------------------------------------

def test_mfma_probe(mxc):
    out = torch.empty(8 * 256, dtype=torch.float32, device="cuda")
    flops = mxc.mxc_probe_mfma(8, 10, out)
    torch.cuda.synchronize()
    assert flops == 8 * 4 * 10 * 4 * 2 * 32 * 32 * 16        # workgroups x waves x iterations x instructions x flops each
    assert torch.isfinite(out).all()
    with pytest.raises(mxc.MxcError):
        mxc.mxc_probe_mfma(16, 10, out)                      # output buffer too small for 16 workgroups


# ---- convolution grouped with bias / ReLU / the ReLU derivative; bias gradient ----------------

FUSED_SHAPES = [
    (2, 16, 10, 11, 24, 3, 3, 1, 1),      # plain matrix-core path, ragged tiles
    (2, 24, 9, 9, 40, 1, 1, 2, 0),        # strided backward-data: zero-filled classes stay zero under the mask
    (1, 3, 22, 24, 8, 11, 11, 4, 2),      # space-to-depth: mask applied by the unpack kernel (16-byte rows)
    (1, 3, 35, 35, 8, 11, 11, 4, 2),      # ... per-pixel unpack
    (1, 2, 12, 15, 8, 5, 5, 2, 2),        # ... dword rows
    (2, 3, 13, 11, 16, 3, 3, 1, 1),       # small-C stride 1: mask applied by the compaction kernel
    (1, 12, 9, 9, 16, 3, 3, 1, 1),        # channel-padded forward
    (2, 5, 13, 13, 7, 5, 5, 1, 2),        # direct kernels
    (1, 136, 6, 5, 264, 3, 3, 1, 1),
]


def _fused_case(dims, dtype, seed):
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy = gen.random_case(seed, *dims, dtype=dtype, dist="normal")
    x = np.maximum(x, 0.0).astype(np.float32)          # the layer below ended in a ReLU: exact zeros and positives
    rng = np.random.Generator(np.random.Philox(key=seed + 99))
    bias = rng.standard_normal(K).astype(np.float32)
    return x, w, dy, bias


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout", ["nhwc", "nchw"])
@pytest.mark.parametrize("dims", FUSED_SHAPES)
def test_grouped_operations(mxc, oracle, dims, dtype, layout):
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy, bias = _fused_case(dims, dtype, hash(dims) & 0xFFFF)
    run = util.Runner(mxc, dims, dtype, layout)
    P, Q = run.P, run.Q
    tb = torch.from_numpy(bias).cuda()
    for relu in (1, 0):
        ref, den = oracle.conv2d_fwd_bias_act(x, w, bias, bool(relu), st, pad)
        y = torch.full((N * K * P * Q,), float("nan"), dtype=run.tdtype, device="cuda")
        mxc.mxc_conv2d_fwd_bias_act(*dims, run.dt, run.lay, run._in(x), run._in(w), tb, relu, y, run._ws(mxc.MXC_FWD))
        got = run._out(y, (N, K, P, Q))
        assert util.metric(got, ref, den) <= util.TOL[dtype], (dims, relu, mxc.mxc_last_variant())
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, dtype, dtype == "bf16")), (dims, relu)
        if relu:
            assert got.min() >= 0.0
    # no bias, no activation: bit-identical to the plain forward
    y0 = run.fwd(x, w, return_tensor=True)
    y1 = torch.empty_like(y0)
    mxc.mxc_conv2d_fwd_bias_act(*dims, run.dt, run.lay, run._in(x), run._in(w), None, 0, y1, run._ws(mxc.MXC_FWD))
    assert torch.equal(y0.view(torch.int16 if dtype == "bf16" else torch.int32), y1.view(torch.int16 if dtype == "bf16" else torch.int32))

    ref, den = oracle.conv2d_bwd_data_relu(dy, w, x, st, pad)
    dx = torch.full((N * C * H * W,), float("nan"), dtype=run.tdtype, device="cuda")
    mxc.mxc_conv2d_bwd_data_relu(*dims, run.dt, run.lay, run._in(dy), run._in(w), run._in(x), dx, run._ws(mxc.MXC_BWD_DATA_RELU))
    got = run._out(dx, (N, C, H, W))
    assert util.metric(got, ref, den) <= util.TOL[dtype], (dims, mxc.mxc_last_variant())
    assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, dtype, dtype == "bf16")), dims
    assert not got[x <= 0].any()

    ref, den = oracle.bias_grad(dy)
    db = torch.full((K,), float("nan"), dtype=torch.float32, device="cuda")
    mxc.mxc_bias_grad(N, K, P, Q, run.dt, run.lay, run._in(dy), db, run._ws(mxc.MXC_BIAS_GRAD))
    got = db.cpu().numpy().astype(np.float64)
    assert util.metric(got, ref, den) <= util.TOL["f32"], dims      # fp32 sums of exact inputs
    db2 = torch.empty_like(db)
    mxc.mxc_bias_grad(N, K, P, Q, run.dt, run.lay, run._in(dy), db2, run._ws(mxc.MXC_BIAS_GRAD))
    assert torch.equal(db.view(torch.int32), db2.view(torch.int32))


PREPARED_SHAPES = [
    (2, 32, 14, 14, 64, 3, 3, 1, 1),       # re-packed filter, one residue class
    (2, 24, 9, 9, 40, 1, 1, 2, 0),         # 1x1 stride 2: transposed filter, classes no tap reaches
    (3, 16, 13, 11, 24, 3, 3, 2, 1),       # four residue classes
    (1, 3, 35, 35, 8, 11, 11, 4, 2),       # space-to-depth first layer
    (1, 3, 20, 18, 16, 3, 3, 1, 1),        # small-C column groups
    (2, 5, 13, 13, 7, 5, 5, 1, 2),         # K % 8 != 0: direct kernel, prepared form is a copy
    (16, 2048, 1, 1, 1024, 1, 1, 1, 0),    # FullyConnected: large 1x1 filter read in place
]


@pytest.mark.parametrize("dtype,layout", [("bf16", "nhwc"), ("bf16", "nchw"), ("f32", "nhwc")])
@pytest.mark.parametrize("dims", PREPARED_SHAPES)
def test_prepared_filter_backward_data(mxc, oracle, dims, dtype, layout):
    """Backward-data from a filter prepared ahead of time: bit-identical to the ordinary entry points (with and
    without the ReLU mask), on repeated use of one prepared buffer, and within the parity bound of the oracle."""
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy, _ = _fused_case(dims, dtype, (hash(dims) & 0xFFFF) + 5)
    run = util.Runner(mxc, dims, dtype, layout)
    d_dy, d_w, d_x = run._in(dy), run._in(w), run._in(x)
    prepared = mxc.alloc_workspace(mxc.mxc_conv2d_workspace_bytes(mxc.MXC_BWD_DATA_FILTER, *dims, run.dt, run.lay))
    mxc.mxc_conv2d_bwd_data_prepare_filter(*dims, run.dt, run.lay, d_w, prepared)
    as_bits = lambda t: t.view(torch.int16 if dtype == "bf16" else torch.int32)
    for mask, op_plain, op_prep in ((None, mxc.MXC_BWD_DATA, mxc.MXC_BWD_DATA_PREPARED),
                                    (d_x, mxc.MXC_BWD_DATA_RELU, mxc.MXC_BWD_DATA_PREPARED_RELU)):
        want = torch.full((N * C * H * W,), float("nan"), dtype=run.tdtype, device="cuda")
        if mask is None:
            mxc.mxc_conv2d_bwd_data(*dims, run.dt, run.lay, d_dy, d_w, want, run._ws(op_plain))
        else:
            mxc.mxc_conv2d_bwd_data_relu(*dims, run.dt, run.lay, d_dy, d_w, mask, want, run._ws(op_plain))
        for _ in range(2):
            got = torch.full_like(want, float("nan"))
            mxc.mxc_conv2d_bwd_data_prepared(*dims, run.dt, run.lay, d_dy, prepared, mask, got, run._ws(op_prep))
            torch.cuda.synchronize()
            assert torch.equal(as_bits(got), as_bits(want)), (dims, dtype, layout, mask is not None, mxc.mxc_last_variant())
    ref, den = oracle.conv2d_bwd_data_relu(dy, w, x, st, pad)
    a = run._out(got, (N, C, H, W))
    assert util.metric(a, ref, den) <= util.TOL[dtype], (dims, mxc.mxc_last_variant())
    assert np.all(np.abs(a - ref) <= util.tight_bound(ref, den, dtype, dtype == "bf16")), dims


PREPARED_INPUT_SHAPES = [
    (2, 3, 67, 67, 16, 11, 11, 4, 2),      # space-to-depth packing (stride 4)
    (2, 3, 33, 35, 24, 7, 7, 2, 3),        # space-to-depth packing (stride 2)
    (2, 3, 30, 30, 16, 3, 3, 1, 1),        # zero-bordered, 4 channels per pixel
    (2, 20, 12, 12, 16, 3, 3, 1, 1),       # channel padding
    (2, 16, 12, 12, 24, 3, 3, 1, 1),       # read as it is: empty prepared form
    (2, 5, 9, 9, 7, 3, 3, 1, 1),           # the two passes use different kernel families: nothing to share, empty form
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("dims", PREPARED_INPUT_SHAPES)
def test_prepared_input_forward_and_backward_weight(mxc, oracle, dims, dtype):
    """Forward (+bias, ReLU) and backward-weight (fp32 and bf16 dw) from one prepared input: bit-identical to the
    ordinary entry points on repeated use of the buffer, and within the parity bound of the oracle."""
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy, bias = _fused_case(dims, dtype, (hash(dims) & 0xFFFF) + 9)
    run = util.Runner(mxc, dims, dtype, "nhwc")
    P, Q = run.P, run.Q
    d_x, d_w, d_dy, d_b = run._in(x), run._in(w), run._in(dy), torch.from_numpy(bias).cuda()
    nbytes = mxc.mxc_conv2d_workspace_bytes(mxc.MXC_INPUT_PREPARED, *dims, run.dt, run.lay)
    assert (nbytes == 0) == (dtype == "f32" or C % 8 == 0 or K % 8 != 0), dims
    prepared = mxc.alloc_workspace(nbytes) if nbytes else None
    mxc.mxc_conv2d_prepare_input(*dims, run.dt, run.lay, d_x, prepared)
    xp = prepared if nbytes else d_x
    as_bits = lambda t: t.view({2: torch.int16, 4: torch.int32}[t.element_size()])
    want = torch.full((N * K * P * Q,), float("nan"), dtype=run.tdtype, device="cuda")
    mxc.mxc_conv2d_fwd_bias_act(*dims, run.dt, run.lay, d_x, d_w, d_b, 1, want, run._ws(mxc.MXC_FWD))
    for _ in range(2):
        got = torch.full_like(want, float("nan"))
        mxc.mxc_conv2d_fwd_prepared_input(*dims, run.dt, run.lay, xp, d_w, d_b, 1, got, run._ws(mxc.MXC_FWD_PREPARED_INPUT))
        torch.cuda.synchronize()
        assert torch.equal(as_bits(got), as_bits(want)), (dims, dtype, mxc.mxc_last_variant())
    ref, den = oracle.conv2d_fwd_bias_act(x, w, bias, True, st, pad)
    a = run._out(got, (N, K, P, Q))
    assert np.all(np.abs(a - ref) <= util.tight_bound(ref, den, dtype, dtype == "bf16")), dims
    cases = [(mxc.MXC_F32, torch.float32, mxc.mxc_conv2d_bwd_weight, mxc.MXC_BWD_WEIGHT, mxc.MXC_BWD_WEIGHT_PREPARED_INPUT)]
    if dtype == "bf16":
        cases.append((mxc.MXC_BF16, torch.bfloat16, mxc.mxc_conv2d_bwd_weight_bf16, mxc.MXC_BWD_WEIGHT_BF16,
                      mxc.MXC_BWD_WEIGHT_PREPARED_INPUT_BF16))
    for dw_dt, tdt, plain_fn, op_plain, op_prep in cases:
        want = torch.full((K * R * S * C,), float("nan"), dtype=tdt, device="cuda")
        plain_fn(*dims, run.dt, run.lay, d_x, d_dy, want, run._ws(op_plain))
        for _ in range(2):
            got = torch.full_like(want, float("nan"))
            mxc.mxc_conv2d_bwd_weight_prepared_input(*dims, run.dt, run.lay, xp, d_dy, got, dw_dt, run._ws(op_prep))
            torch.cuda.synchronize()
            assert torch.equal(as_bits(got), as_bits(want)), (dims, dtype, dw_dt, mxc.mxc_last_variant())
        if dw_dt == mxc.MXC_F32:
            ref = oracle.conv2d_bwd_weight(x, dy, w.shape, st, pad)
            den = oracle.conv2d_bwd_weight(np.abs(x), np.abs(dy), w.shape, st, pad)
            a = util.nhwc_to_nchw(got.cpu().numpy().astype(np.float64).reshape(K, R, S, C))
            assert util.metric(a, ref, den) <= util.TOL[dtype], (dims, mxc.mxc_last_variant())


TRANSFORM_SHAPES = [
    (2, 16, 12, 12, 24, 3, 3, 1, 1),
    (1, 64, 13, 15, 72, 3, 3, 1, 1),       # odd output sizes: half-filled blocks at the right and bottom edges
    (2, 8, 9, 10, 16, 3, 3, 1, 0),         # no padding
    (1, 16, 6, 6, 8, 3, 3, 1, 2),          # output larger than the input
    (2, 128, 28, 28, 128, 3, 3, 1, 1),     # several row and column tiles of the GEMMs
]


@pytest.mark.parametrize("dims", TRANSFORM_SHAPES)
def test_transform_domain_forward(mxc, oracle, dims):
    """The 3x3 stride-1 forward evaluated in the transform domain, against the plain definition: inside the
    spec tolerance, and inside its own budget - 2^-8 times the worst-case weight of its two bf16 roundings
    (evaluated on the host from the transform's definition), plus the rounding of the result."""
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy, bias = _fused_case(dims, "bf16", (hash(dims) & 0xFFFF) + 13)
    run = util.Runner(mxc, dims, "bf16", "nhwc")
    P, Q = run.P, run.Q
    d_x, d_w, d_b = run._in(x), run._in(w), torch.from_numpy(bias).cuda()
    ws = mxc.alloc_workspace(mxc.mxc_conv2d_workspace_bytes(mxc.MXC_FWD_TRANSFORM, *dims, run.dt, run.lay))
    budget = util.transform_domain_budget(x, w, pad)
    for b, relu in ((None, 0), (d_b, 1)):
        y = torch.full((N * K * P * Q,), float("nan"), dtype=torch.bfloat16, device="cuda")
        mxc.mxc_conv2d_fwd_transform(*dims, run.dt, run.lay, d_x, d_w, b, relu, y, ws)
        torch.cuda.synchronize()
        assert mxc.mxc_last_variant().startswith("fwd:winograd"), mxc.mxc_last_variant()
        got = run._out(y, (N, K, P, Q))
        if b is None:
            ref, den = oracle.conv2d_fwd(x, w, st, pad), oracle.conv2d_fwd(np.abs(x), np.abs(w), st, pad)
        else:
            ref, den = oracle.conv2d_fwd_bias_act(x, w, bias, True, st, pad)
        assert util.metric(got, ref, den) <= util.TOL["bf16"], dims
        bound = 2.0 ** -8 * 1.05 * budget + 2.0 ** -8 * np.abs(ref) + 64 * 2.0 ** -24 * den
        assert np.all(np.abs(got - ref) <= bound), (dims, float(np.max(np.abs(got - ref) / np.maximum(bound, 1e-30))))
    # the direct form on the same inputs, for the record of how much wider the budget is used
    yd = torch.empty_like(y)
    mxc.mxc_conv2d_fwd_bias_act(*dims, run.dt, run.lay, d_x, d_w, d_b, 1, yd, run._ws(mxc.MXC_FWD))
    torch.cuda.synchronize()
    assert util.metric(run._out(yd, (N, K, P, Q)), ref, den) <= util.metric(got, ref, den) + 1e-3


@pytest.mark.parametrize("cfg_idx", [1, 3])
def test_grouped_operations_network_layers(mxc, oracle, cfg_idx):
    """The bench's launch configuration (bf16, NHWC) on every layer of the AlexNet- and VGG-style stacks, batch 2."""
    cfg = gen.CONFIGS[cfg_idx]
    for li in range(len(cfg.layers)):
        L, t = gen.layer_inputs(cfg, li, batch=1 if cfg.layers[li].H >= 112 else 2)
        dims = L.dims()
        N, C, H, W, K, R, S, st, pad = dims
        x = np.maximum(t["x"], 0.0).astype(np.float32)
        w, dy = t["w"], t["dy"]
        bias = np.linspace(-1.0, 1.0, K).astype(np.float32)
        run = util.Runner(mxc, dims, "bf16", "nhwc")
        ref, den = oracle.conv2d_fwd_bias_act(x, w, bias, True, st, pad)
        y = torch.full((N * K * L.P * L.Q,), float("nan"), dtype=torch.bfloat16, device="cuda")
        mxc.mxc_conv2d_fwd_bias_act(*dims, run.dt, run.lay, run._in(x), run._in(w), torch.from_numpy(bias).cuda(), 1, y, run._ws(mxc.MXC_FWD))
        got = run._out(y, (N, K, L.P, L.Q))
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True)), L.name
        ref, den = oracle.conv2d_bwd_data_relu(dy, w, x, st, pad)
        dx = torch.full((N * C * H * W,), float("nan"), dtype=torch.bfloat16, device="cuda")
        mxc.mxc_conv2d_bwd_data_relu(*dims, run.dt, run.lay, run._in(dy), run._in(w), run._in(x), dx, run._ws(mxc.MXC_BWD_DATA_RELU))
        got = run._out(dx, (N, C, H, W))
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True)), L.name
        ref, den = oracle.bias_grad(dy)
        db = torch.empty(K, dtype=torch.float32, device="cuda")
        mxc.mxc_bias_grad(N, K, L.P, L.Q, run.dt, run.lay, run._in(dy), db, run._ws(mxc.MXC_BIAS_GRAD))
        assert util.metric(db.cpu().numpy().astype(np.float64), ref, den) <= util.TOL["f32"], L.name


# ---- weight update ------------------------------------------------------------------------------

@pytest.mark.parametrize("n", [1, 3, 1024, 4099, 884736 + 3])
@pytest.mark.parametrize("momentum,wd", [(0.0, 0.0), (0.9, 1e-4)])
def test_sgd_update(mxc, oracle, n, momentum, wd):
    rng = np.random.Generator(np.random.Philox(key=gen.SEED + n))
    w0 = rng.standard_normal(n).astype(np.float32)
    gs = [rng.standard_normal(n).astype(np.float32) for _ in range(3)]
    w = torch.from_numpy(w0).cuda()
    v = torch.zeros(n, dtype=torch.float32, device="cuda") if momentum else None
    wb = torch.full((n,), float("nan"), dtype=torch.bfloat16, device="cuda")
    rw, rv = w0.astype(np.float64), None
    for g in gs:
        mxc.mxc_sgd_update(w, torch.from_numpy(g).cuda(), v, wb, 0.05, momentum, wd)
        rw, rv = oracle.sgd_update(rw, g, rv, 0.05, momentum, wd)
    torch.cuda.synchronize()
    got = w.cpu().numpy().astype(np.float64)
    scale = np.abs(rw) + sum(0.05 * np.abs(g.astype(np.float64)) for g in gs) + 1e-30
    assert np.max(np.abs(got - rw) / scale) <= 1e-6          # a handful of fp32 roundings per step
    if momentum:
        assert np.max(np.abs(v.cpu().numpy() - rv) / scale) <= 1e-6
    # the bf16 copy is the fp32 master rounded to nearest even, bit for bit
    assert np.array_equal(gen.to_host_f64(wb), gen.round_to_bf16(w.cpu().numpy()).astype(np.float64))
    with pytest.raises(mxc.MxcError):
        mxc.mxc_sgd_update(w, torch.from_numpy(gs[0]).cuda(), None, None, 0.05, 0.9, 0.0)    # momentum without velocity


# ---- split reduction (few tiles, long reduction: FullyConnected-shaped and small-batch problems) -----

SPLIT_SHAPES = [
    (64, 2048, 1, 1, 256, 1, 1, 1, 0),      # FullyConnected: one row tile, 32 stages
    (128, 1024, 1, 1, 520, 1, 1, 1, 0),     # ... ragged output columns
    (1, 256, 14, 14, 128, 3, 3, 1, 1),      # one image: two row tiles (ragged), 36 stages, channel-block-major order
    (2, 192, 7, 7, 64, 5, 5, 1, 2),         # 75 stages, ragged last split
    (3, 136, 5, 5, 32, 3, 3, 1, 1),         # channel count not a multiple of 64: tap-major order
]


@pytest.mark.parametrize("dims", SPLIT_SHAPES)
def test_split_reduction_forward(mxc, oracle, dims):
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy, bias = _fused_case(dims, "bf16", hash(dims) & 0xFFFF)
    check_all_passes(mxc, oracle, dims, "bf16", "nhwc", x, w, dy, passes=("fwd",))
    run = util.Runner(mxc, dims, "bf16", "nhwc")
    y = run.fwd(x, w, return_tensor=True)
    assert "_split" in mxc.mxc_last_variant(), mxc.mxc_last_variant()
    assert torch.equal(y.view(torch.int16), run.fwd(x, w, return_tensor=True).view(torch.int16))      # deterministic
    # bias and ReLU are applied by the finishing kernel
    ref, den = oracle.conv2d_fwd_bias_act(x, w, bias, True, st, pad)
    y = torch.full((N * K * run.P * run.Q,), float("nan"), dtype=torch.bfloat16, device="cuda")
    mxc.mxc_conv2d_fwd_bias_act(*dims, run.dt, run.lay, run._in(x), run._in(w), torch.from_numpy(bias).cuda(), 1, y, run._ws(mxc.MXC_FWD))
    got = run._out(y, (N, K, run.P, run.Q))
    assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True)), dims


@pytest.mark.parametrize("dims", [(64, 256, 1, 1, 2048, 1, 1, 1, 0), (128, 520, 1, 1, 1024, 1, 1, 1, 0),
                                  (64, 2048, 1, 1, 1024, 1, 1, 1, 0),       # 4 MB filter: read in place (transposed tiles)
                                  (32, 2056, 1, 1, 1024, 1, 1, 1, 0)]       # ... ragged output columns
                         + SPLIT_SHAPES[2:4])
def test_split_reduction_backward_data(mxc, oracle, dims):
    N, C, H, W, K, R, S, st, pad = dims
    x, w, dy, _ = _fused_case(dims, "bf16", (hash(dims) + 5) & 0xFFFF)
    check_all_passes(mxc, oracle, dims, "bf16", "nhwc", x, w, dy, passes=("bwd_data",))
    run = util.Runner(mxc, dims, "bf16", "nhwc")
    a = run.bwd_data(dy, w, return_tensor=True)
    assert "_split" in mxc.mxc_last_variant(), mxc.mxc_last_variant()
    assert torch.equal(a.view(torch.int16), run.bwd_data(dy, w, return_tensor=True).view(torch.int16))
    ref, den = oracle.conv2d_bwd_data_relu(dy, w, x, st, pad)
    dx = torch.full((N * C * H * W,), float("nan"), dtype=torch.bfloat16, device="cuda")
    mxc.mxc_conv2d_bwd_data_relu(*dims, run.dt, run.lay, run._in(dy), run._in(w), run._in(x), dx, run._ws(mxc.MXC_BWD_DATA_RELU))
    got = run._out(dx, (N, C, H, W))
    assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, "bf16", True)), dims
    assert not got[x <= 0].any()


# ---- FullyConnected entry points --------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("N,C,K", [(128, 1024, 512), (64, 2048, 264), (5, 24, 40), (32, 136, 72), (256, 64, 16), (128, 4096, 512)])
def test_fully_connected(mxc, oracle, N, C, K, dtype):
    rng = np.random.Generator(np.random.Philox(key=gen.SEED + N * C + K))
    rnd = lambda *shape: (gen.round_to_bf16(rng.standard_normal(shape).astype(np.float32)) if dtype == "bf16"
                          else rng.standard_normal(shape).astype(np.float32))
    x = np.maximum(rnd(N, C), 0.0).astype(np.float32)
    w, dy = rnd(K, C) * np.float32(0.125), rnd(N, K)
    w = gen.round_to_bf16(w) if dtype == "bf16" else w
    bias = rng.standard_normal(K).astype(np.float32)
    dt = mxc.MXC_BF16 if dtype == "bf16" else mxc.MXC_F32
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    dims = (N, C, 1, 1, K, 1, 1, 1, 0)
    ws = lambda op: mxc.alloc_workspace(mxc.mxc_conv2d_workspace_bytes(op, *dims, dt, mxc.MXC_NHWC))
    dev = lambda a: gen.to_device(a, dtype)
    out_bf16 = dtype == "bf16"

    y = torch.full((N * K,), float("nan"), dtype=td, device="cuda")
    mxc.mxc_fc_fwd(N, C, K, dt, dev(x), dev(w), torch.from_numpy(bias).cuda(), 1, y, ws(mxc.MXC_FWD))
    ref, den = oracle.fc_fwd(x, w, bias, True)
    got = gen.to_host_f64(y).reshape(N, K)
    assert util.metric(got, ref, den) <= util.TOL[dtype]
    assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, dtype, out_bf16))

    for mask in (None, x):
        dx = torch.full((N * C,), float("nan"), dtype=td, device="cuda")
        mxc.mxc_fc_bwd_data(N, C, K, dt, dev(dy), dev(w), None if mask is None else dev(mask), dx, ws(mxc.MXC_BWD_DATA_RELU))
        ref, den = oracle.fc_bwd_data(dy, w, mask)
        got = gen.to_host_f64(dx).reshape(N, C)
        assert util.metric(got, ref, den) <= util.TOL[dtype]
        assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, dtype, out_bf16))

    dw = torch.full((K * C,), float("nan"), dtype=torch.float32, device="cuda")
    mxc.mxc_fc_bwd_weight(N, C, K, dt, dev(x), dev(dy), dw, ws(mxc.MXC_BWD_WEIGHT))
    ref, den = oracle.fc_bwd_weight(x, dy)
    got = dw.cpu().numpy().astype(np.float64).reshape(K, C)
    assert util.metric(got, ref, den) <= util.TOL[dtype]
    assert np.all(np.abs(got - ref) <= util.tight_bound(ref, den, dtype, False))


# ---- softmax output layer -----------------------------------------------------------------------

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N,K", [(1, 1), (3, 10), (128, 1000), (7, 4099)])
def test_softmax(mxc, oracle, N, K, dtype):
    rng = np.random.Generator(np.random.Philox(key=gen.SEED + 13 * N + K))
    z = (rng.standard_normal((N, K)) * 4).astype(np.float32)
    if dtype == "bf16":
        z = gen.round_to_bf16(z)
    labels = rng.integers(0, K, size=N).astype(np.int32)
    dt = mxc.MXC_BF16 if dtype == "bf16" else mxc.MXC_F32
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    p = torch.full((N * K,), float("nan"), dtype=td, device="cuda")
    mxc.mxc_softmax_fwd(N, K, dt, gen.to_device(z, dtype), p)
    got = gen.to_host_f64(p).reshape(N, K)
    ref = oracle.softmax_fwd(z)
    # fp32 exp and a sum of K terms, then one rounding to the storage type
    tol = 2.0 ** -8 if dtype == "bf16" else 1e-5
    assert np.all(np.abs(got - ref) <= tol * ref + 1e-30)
    dz = torch.full((N * K,), float("nan"), dtype=td, device="cuda")
    mxc.mxc_softmax_xent_bwd(N, K, dt, p, torch.from_numpy(labels).cuda(), 0.5, dz)
    gotg = gen.to_host_f64(dz).reshape(N, K)
    refg = oracle.softmax_xent_bwd(got, labels, 0.5)          # from the probabilities the GPU stored
    assert np.all(np.abs(gotg - refg) <= (2.0 ** -8 if dtype == "bf16" else 1e-6) * np.abs(refg) + 1e-30)

