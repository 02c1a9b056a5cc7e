"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, validates arguments before touching the device, and answers workspace queries."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mxc.h")


@pytest.fixture(scope="module")
def mxc():
    from paper_1512_01274_amd import mxc as m
    return m


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mxc_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(mxc):
    names = declared_symbols()
    assert {"mxc_conv2d_fwd", "mxc_conv2d_bwd_data", "mxc_conv2d_bwd_weight", "mxc_conv2d_workspace_bytes",
            "mxc_layout_convert", "mxc_status_string", "mxc_last_variant", "mxc_version"} <= set(names)
    lib = ctypes.CDLL(mxc.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    for n in names:
        assert hasattr(mxc, n), f"binding lacks {n}"


def test_status_strings(mxc):
    seen = set()
    for code in range(0, 7):
        s = mxc.mxc_status_string(code)
        assert s and s != "unknown status" and s not in seen
        seen.add(s)
    assert mxc.mxc_status_string(99) == "unknown status"
    assert mxc.mxc_version() >= 100
    assert isinstance(mxc.mxc_last_variant(), str)


GOOD = (2, 16, 16, 16, 32, 3, 3, 1, 1)


@pytest.mark.parametrize("pos,val", [(0, 0), (1, -1), (2, 0), (3, 0), (4, 0), (5, 0), (6, -2), (7, 0), (8, -1),
                                     (5, 19), (6, 19)])
def test_shape_errors_before_any_pointer_use(mxc, pos, val):
    dims = list(GOOD)
    dims[pos] = val
    lib = mxc.raw()
    for fn in (lib.mxc_conv2d_fwd, lib.mxc_conv2d_bwd_data, lib.mxc_conv2d_bwd_weight):
        assert fn(*dims, mxc.MXC_F32, mxc.MXC_NCHW, None, None, None, None, 0, None) == mxc.MXC_ERR_SHAPE
    with pytest.raises(mxc.MxcError) as e:
        mxc.mxc_conv2d_workspace_bytes(mxc.MXC_FWD, *dims, mxc.MXC_F32, mxc.MXC_NCHW)
    assert e.value.status == mxc.MXC_ERR_SHAPE


def test_unsupported_and_null(mxc):
    lib = mxc.raw()
    assert lib.mxc_conv2d_fwd(*GOOD, 7, mxc.MXC_NCHW, None, None, None, None, 0, None) == mxc.MXC_ERR_UNSUPPORTED
    assert lib.mxc_conv2d_fwd(*GOOD, mxc.MXC_BF16, 5, None, None, None, None, 0, None) == mxc.MXC_ERR_UNSUPPORTED
    assert lib.mxc_conv2d_fwd(*GOOD, mxc.MXC_BF16, mxc.MXC_NHWC, None, None, None, None, 0, None) == mxc.MXC_ERR_NULL
    assert lib.mxc_conv2d_fwd(*GOOD, mxc.MXC_BF16, mxc.MXC_NHWC, 4096, 8192, None, None, 0, None) == mxc.MXC_ERR_NULL
    # misaligned (fake, never dereferenced) pointers are rejected before any launch
    assert lib.mxc_conv2d_bwd_data(*GOOD, mxc.MXC_BF16, mxc.MXC_NHWC, 4096, 8192 + 2, 16384, None, 0, None) \
        == mxc.MXC_ERR_ALIGN
    assert lib.mxc_layout_convert(1, 2, 3, 4, mxc.MXC_F32, 0, 1, None, None, None) == mxc.MXC_ERR_NULL
    assert lib.mxc_layout_convert(0, 2, 3, 4, mxc.MXC_F32, 0, 1, None, None, None) == mxc.MXC_ERR_SHAPE
    assert lib.mxc_layout_convert(1, 2, 3, 4, 9, 0, 1, None, None, None) == mxc.MXC_ERR_UNSUPPORTED
    assert lib.mxc_conv2d_workspace_bytes(9, *GOOD, 0, 0, ctypes.byref(ctypes.c_size_t())) == mxc.MXC_ERR_UNSUPPORTED
    assert lib.mxc_conv2d_workspace_bytes(0, *GOOD, 0, 0, None) == mxc.MXC_ERR_NULL


def test_workspace_query_is_consistent(mxc):
    for op in (mxc.MXC_FWD, mxc.MXC_BWD_DATA, mxc.MXC_BWD_WEIGHT):
        for dt in (mxc.MXC_F32, mxc.MXC_BF16):
            nchw = mxc.mxc_conv2d_workspace_bytes(op, *GOOD, dt, mxc.MXC_NCHW)
            nhwc = mxc.mxc_conv2d_workspace_bytes(op, *GOOD, dt, mxc.MXC_NHWC)
            assert nchw % 256 == 0 and nhwc % 256 == 0
            # NCHW needs room for the converted copies of all three tensors on top of the NHWC need
            assert nchw > nhwc
    # a call with too small a workspace is refused on the host, before any launch (fake aligned pointers)
    lib = mxc.raw()
    need = mxc.mxc_conv2d_workspace_bytes(mxc.MXC_FWD, *GOOD, mxc.MXC_F32, mxc.MXC_NCHW)
    assert lib.mxc_conv2d_fwd(*GOOD, mxc.MXC_F32, mxc.MXC_NCHW, 4096, 8192, 16384, 32768, need - 1, None) \
        == mxc.MXC_ERR_WORKSPACE
