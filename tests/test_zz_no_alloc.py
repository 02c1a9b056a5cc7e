"""The backward-weight entry point that allocates nothing (its split-reduction scratch is an array in
the library's device code) against the ordinary entry point, through the C ABI: two calls in a row,
the second with a smaller input, results bit-identical (both run the same kernels in the same
order), and the ordinary entry point's own parity against the oracle is covered by the other tests.
Also: a problem whose scratch need exceeds the array is rejected before anything runs."""
import ctypes

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


def _both(mxc, oracle, dims, dtype, layout, seed):
    N, C, H, W, K, R, S, st, pad = dims
    P, Q = (H + 2 * pad - R) // st + 1, (W + 2 * pad - S) // st + 1
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    dy = rng.standard_normal((N, K, P, Q)).astype(np.float32)
    if dtype == "bf16":
        x, dy = gen.round_to_bf16(x), gen.round_to_bf16(dy)
    run = util.Runner(mxc, dims, dtype, layout)
    dx_, ddy = run._in(x), run._in(dy)
    want = torch.full((K * C * R * S,), float("nan"), dtype=torch.float32, device="cuda")
    got = torch.full_like(want, float("nan"))
    mxc.mxc_conv2d_bwd_weight(*dims, run.dt, run.lay, dx_, ddy, want, run._ws(mxc.MXC_BWD_WEIGHT))
    # through the raw C ABI: plain pointers and sizes, no workspace argument
    rc = mxc.raw().mxc_conv2d_bwd_weight_static(*dims, run.dt, run.lay, ctypes.c_void_p(dx_.data_ptr()),
                                                ctypes.c_void_p(ddy.data_ptr()), ctypes.c_void_p(got.data_ptr()),
                                                ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == mxc.MXC_OK, mxc.mxc_status_string(rc)
    torch.cuda.synchronize()
    assert torch.equal(got, want), f"{dims} {dtype} {layout}: static-scratch result differs from the workspace result"
    # and against the oracle, to the parity tests' bar
    a = got.cpu().numpy().astype(np.float64)
    a = util.nhwc_to_nchw(a.reshape(K, R, S, C)) if layout == "nhwc" else a.reshape(K, C, R, S)
    ref = oracle.conv2d_bwd_weight(x, dy, (K, C, R, S), st, pad)
    den = oracle.conv2d_bwd_weight(np.abs(x), np.abs(dy), (K, C, R, S), st, pad)
    assert util.metric(a, ref, den) <= util.TOL[dtype]
    assert (np.abs(a - ref) <= util.tight_bound(ref, den, dtype, False)).all()


@pytest.mark.parametrize("dtype,layout", [("bf16", "nhwc"), ("bf16", "nchw"), ("f32", "nhwc")])
def test_static_scratch_matches_workspace_entry_twice(mxc, oracle, dtype, layout):
    # first call: many splits of a ragged problem; second call: a smaller input, which leaves most of the
    # first call's partial sums in the array
    _both(mxc, oracle, (6, 72, 19, 17, 104, 3, 3, 1, 1), dtype, layout, seed=11)
    _both(mxc, oracle, (2, 24, 9, 9, 40, 3, 3, 2, 1), dtype, layout, seed=12)
    # and once more the first shape: a stale smaller result must not leak into it
    _both(mxc, oracle, (6, 72, 19, 17, 104, 3, 3, 1, 1), dtype, layout, seed=13)


def test_static_scratch_rejects_oversize(mxc):
    # VGG conv1_1 in NCHW needs both operands converted through the scratch: far beyond 64 MiB
    dims = (64, 3, 224, 224, 64, 3, 3, 1, 1)
    need = mxc.mxc_conv2d_workspace_bytes(mxc.MXC_BWD_WEIGHT, *dims, mxc.MXC_BF16, mxc.MXC_NCHW)
    assert need > (64 << 20)
    t = torch.zeros(64, dtype=torch.bfloat16, device="cuda")     # never touched: the size check comes first
    rc = mxc.raw().mxc_conv2d_bwd_weight_static(*dims, mxc.MXC_BF16, mxc.MXC_NCHW, ctypes.c_void_p(t.data_ptr()),
                                                ctypes.c_void_p(t.data_ptr()), ctypes.c_void_p(t.data_ptr()), None)
    assert rc == mxc.MXC_ERR_WORKSPACE
