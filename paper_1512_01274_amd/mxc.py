"""ctypes binding over libmxc.so: argument marshalling only.

Function names and argument order mirror include/mxc.h.  Tensors are torch
tensors on the GPU (torch is used for device memory and streams, nothing else);
every step of the computation runs in the library's HIP kernels.  There is no
CPU or PyTorch fallback: if the library cannot be loaded, importing this module
raises.
"""
import ctypes
import os

import torch

MXC_OK = 0
MXC_ERR_NULL, MXC_ERR_SHAPE, MXC_ERR_UNSUPPORTED, MXC_ERR_WORKSPACE, MXC_ERR_ALIGN, MXC_ERR_LAUNCH = 1, 2, 3, 4, 5, 6
MXC_F32, MXC_BF16 = 0, 1
MXC_NCHW, MXC_NHWC = 0, 1
MXC_FWD, MXC_BWD_DATA, MXC_BWD_WEIGHT, MXC_BWD_DATA_RELU, MXC_BIAS_GRAD = 0, 1, 2, 3, 4
MXC_BWD_DATA_FILTER, MXC_BWD_DATA_PREPARED, MXC_BWD_DATA_PREPARED_RELU, MXC_BWD_WEIGHT_BF16 = 5, 6, 7, 8
MXC_INPUT_PREPARED, MXC_FWD_PREPARED_INPUT, MXC_BWD_WEIGHT_PREPARED_INPUT, MXC_BWD_WEIGHT_PREPARED_INPUT_BF16 = 9, 10, 11, 12
MXC_FWD_TRANSFORM = 13

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmxc.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1512_01274_amd.build`")
_lib = ctypes.CDLL(LIB_PATH)

_I, _VP, _SZ = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
for _name in ("mxc_conv2d_fwd", "mxc_conv2d_bwd_data", "mxc_conv2d_bwd_weight", "mxc_conv2d_bwd_weight_bf16"):
    _f = getattr(_lib, _name)
    _f.argtypes = [_I] * 11 + [_VP, _VP, _VP, _VP, _SZ, _VP]
    _f.restype = _I
_lib.mxc_conv2d_bwd_weight_static.argtypes = [_I] * 11 + [_VP, _VP, _VP, _VP]
_lib.mxc_conv2d_bwd_weight_static.restype = _I
_lib.mxc_conv2d_bwd_data_prepare_filter.argtypes = [_I] * 11 + [_VP, _VP, _SZ, _VP]
_lib.mxc_conv2d_bwd_data_prepare_filter.restype = _I
_lib.mxc_conv2d_bwd_data_prepared.argtypes = [_I] * 11 + [_VP, _VP, _SZ, _VP, _VP, _VP, _SZ, _VP]
_lib.mxc_conv2d_bwd_data_prepared.restype = _I
_lib.mxc_conv2d_prepare_input.argtypes = [_I] * 11 + [_VP, _VP, _SZ, _VP]
_lib.mxc_conv2d_prepare_input.restype = _I
_lib.mxc_conv2d_fwd_prepared_input.argtypes = [_I] * 11 + [_VP, _SZ, _VP, _VP, _I, _VP, _VP, _SZ, _VP]
_lib.mxc_conv2d_fwd_prepared_input.restype = _I
_lib.mxc_conv2d_bwd_weight_prepared_input.argtypes = [_I] * 11 + [_VP, _SZ, _VP, _VP, _I, _VP, _SZ, _VP]
_lib.mxc_conv2d_bwd_weight_prepared_input.restype = _I
_lib.mxc_conv2d_fwd_transform.argtypes = [_I] * 11 + [_VP, _VP, _VP, _I, _VP, _VP, _SZ, _VP]
_lib.mxc_conv2d_fwd_transform.restype = _I
_lib.mxc_conv2d_workspace_bytes.argtypes = [_I] * 12 + [ctypes.POINTER(_SZ)]
_lib.mxc_conv2d_workspace_bytes.restype = _I
_lib.mxc_layout_convert.argtypes = [_I] * 7 + [_VP, _VP, _VP]
_lib.mxc_layout_convert.restype = _I
_lib.mxc_status_string.argtypes = [_I]
_lib.mxc_status_string.restype = ctypes.c_char_p
_lib.mxc_last_variant.argtypes = []
_lib.mxc_last_variant.restype = ctypes.c_char_p
_lib.mxc_version.argtypes = []
_lib.mxc_version.restype = _I
_lib.mxc_tile_name.argtypes = [_I, _I]
_lib.mxc_tile_name.restype = ctypes.c_char_p
_lib.mxc_conv2d_fwd_bias_act.argtypes = [_I] * 11 + [_VP, _VP, _VP, _I, _VP, _VP, _SZ, _VP]
_lib.mxc_conv2d_fwd_bias_act.restype = _I
_lib.mxc_conv2d_bwd_data_relu.argtypes = [_I] * 11 + [_VP, _VP, _VP, _VP, _VP, _SZ, _VP]
_lib.mxc_conv2d_bwd_data_relu.restype = _I
_lib.mxc_bias_grad.argtypes = [_I] * 6 + [_VP, _VP, _VP, _SZ, _VP]
_lib.mxc_bias_grad.restype = _I
_lib.mxc_fc_fwd.argtypes = [_I] * 4 + [_VP, _VP, _VP, _I, _VP, _VP, _SZ, _VP]
_lib.mxc_fc_fwd.restype = _I
_lib.mxc_fc_bwd_data.argtypes = [_I] * 4 + [_VP, _VP, _VP, _VP, _VP, _SZ, _VP]
_lib.mxc_fc_bwd_data.restype = _I
_lib.mxc_fc_bwd_weight.argtypes = [_I] * 4 + [_VP, _VP, _VP, _VP, _SZ, _VP]
_lib.mxc_fc_bwd_weight.restype = _I
_lib.mxc_softmax_fwd.argtypes = [_I, _I, _I, _VP, _VP, _VP]
_lib.mxc_softmax_fwd.restype = _I
_lib.mxc_softmax_xent_bwd.argtypes = [_I, _I, _I, _VP, _VP, ctypes.c_float, _VP, _VP]
_lib.mxc_softmax_xent_bwd.restype = _I
_F = ctypes.c_float
_lib.mxc_sgd_update.argtypes = [_SZ, _VP, _VP, _VP, _VP, _F, _F, _F, _VP]
_lib.mxc_sgd_update.restype = _I
_lib.mxc_probe_mfma.argtypes = [_I, _I, _VP, _SZ, ctypes.POINTER(ctypes.c_double), _VP]
_lib.mxc_probe_mfma.restype = _I


class MxcError(RuntimeError):
    def __init__(self, status):
        self.status = status
        super().__init__(f"mxc status {status}: {mxc_status_string(status)}")


def mxc_status_string(status: int) -> str:
    return _lib.mxc_status_string(status).decode()


def mxc_last_variant() -> str:
    return _lib.mxc_last_variant().decode()


def mxc_version() -> int:
    return _lib.mxc_version()


def mxc_tile_name(family: int, index: int):
    n = _lib.mxc_tile_name(family, index)
    return None if n is None else n.decode()


_lib.mxc_last_plan_key.argtypes = [ctypes.POINTER(ctypes.c_longlong), ctypes.POINTER(_I), ctypes.POINTER(_I)]
_lib.mxc_last_plan_key.restype = None


def mxc_last_plan_key():
    """(M, Co, Kd) of the implicit GEMM the last forward / backward-data call of this thread planned."""
    m, co, kd = ctypes.c_longlong(0), _I(0), _I(0)
    _lib.mxc_last_plan_key(ctypes.byref(m), ctypes.byref(co), ctypes.byref(kd))
    return m.value, co.value, kd.value


def mxc_tile_names(family: int):
    """Names of the tile shapes of a kernel family (0: implicit GEMM, 1: backward-weight, 2: the streaming and the window implicit GEMM)."""
    out, i = [], 0
    while True:
        n = _lib.mxc_tile_name(family, i)
        if n is None:
            return out
        out.append(n.decode())
        i += 1


def dtype_code(t: torch.dtype) -> int:
    if t == torch.float32:
        return MXC_F32
    if t == torch.bfloat16:
        return MXC_BF16
    raise TypeError(f"unsupported dtype {t}")


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous GPU tensors")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def mxc_conv2d_workspace_bytes(op, N, C, H, W, K, R, S, stride, pad, dtype, layout) -> int:
    out = _SZ(0)
    rc = _lib.mxc_conv2d_workspace_bytes(op, N, C, H, W, K, R, S, stride, pad, dtype, layout, ctypes.byref(out))
    if rc != MXC_OK:
        raise MxcError(rc)
    return int(out.value)


def _call(fn, dims, dtype, layout, a, b, out, workspace, stream):
    ws_ptr = _ptr(workspace) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    rc = fn(*dims, dtype, layout, _ptr(a), _ptr(b), _ptr(out), ws_ptr, ws_bytes, _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_conv2d_fwd(N, C, H, W, K, R, S, stride, pad, dtype, layout, x, w, y, workspace=None, stream=None):
    _call(_lib.mxc_conv2d_fwd, (N, C, H, W, K, R, S, stride, pad), dtype, layout, x, w, y, workspace, stream)


def mxc_conv2d_bwd_data(N, C, H, W, K, R, S, stride, pad, dtype, layout, dy, w, dx, workspace=None, stream=None):
    _call(_lib.mxc_conv2d_bwd_data, (N, C, H, W, K, R, S, stride, pad), dtype, layout, dy, w, dx, workspace, stream)


def mxc_conv2d_bwd_weight(N, C, H, W, K, R, S, stride, pad, dtype, layout, x, dy, dw, workspace=None, stream=None):
    _call(_lib.mxc_conv2d_bwd_weight, (N, C, H, W, K, R, S, stride, pad), dtype, layout, x, dy, dw, workspace, stream)


def mxc_conv2d_bwd_weight_bf16(N, C, H, W, K, R, S, stride, pad, dtype, layout, x, dy, dw, workspace=None, stream=None):
    _call(_lib.mxc_conv2d_bwd_weight_bf16, (N, C, H, W, K, R, S, stride, pad), dtype, layout, x, dy, dw, workspace, stream)


def mxc_conv2d_bwd_weight_static(N, C, H, W, K, R, S, stride, pad, dtype, layout, x, dy, dw, stream=None):
    rc = _lib.mxc_conv2d_bwd_weight_static(N, C, H, W, K, R, S, stride, pad, dtype, layout, _ptr(x), _ptr(dy), _ptr(dw),
                                           _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def _ws(workspace):
    if workspace is None:
        return None, 0
    return _ptr(workspace), workspace.numel() * workspace.element_size()


def mxc_conv2d_fwd_bias_act(N, C, H, W, K, R, S, stride, pad, dtype, layout, x, w, bias, relu, y, workspace=None, stream=None):
    ws_ptr, ws_bytes = _ws(workspace)
    rc = _lib.mxc_conv2d_fwd_bias_act(N, C, H, W, K, R, S, stride, pad, dtype, layout, _ptr(x), _ptr(w), _ptr(bias), int(relu),
                                      _ptr(y), ws_ptr, ws_bytes, _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_conv2d_bwd_data_relu(N, C, H, W, K, R, S, stride, pad, dtype, layout, dy, w, x, dx, workspace=None, stream=None):
    ws_ptr, ws_bytes = _ws(workspace)
    rc = _lib.mxc_conv2d_bwd_data_relu(N, C, H, W, K, R, S, stride, pad, dtype, layout, _ptr(dy), _ptr(w), _ptr(x), _ptr(dx),
                                       ws_ptr, ws_bytes, _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_conv2d_bwd_data_prepare_filter(N, C, H, W, K, R, S, stride, pad, dtype, layout, w, w_prepared, stream=None):
    rc = _lib.mxc_conv2d_bwd_data_prepare_filter(N, C, H, W, K, R, S, stride, pad, dtype, layout, _ptr(w), _ptr(w_prepared),
                                                 w_prepared.numel() * w_prepared.element_size(), _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_conv2d_bwd_data_prepared(N, C, H, W, K, R, S, stride, pad, dtype, layout, dy, w_prepared, x_mask, dx, workspace=None,
                                 stream=None):
    ws_ptr, ws_bytes = _ws(workspace)
    rc = _lib.mxc_conv2d_bwd_data_prepared(N, C, H, W, K, R, S, stride, pad, dtype, layout, _ptr(dy), _ptr(w_prepared),
                                           w_prepared.numel() * w_prepared.element_size(), _ptr(x_mask), _ptr(dx), ws_ptr, ws_bytes,
                                           _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_conv2d_fwd_transform(N, C, H, W, K, R, S, stride, pad, dtype, layout, x, w, bias, relu, y, workspace=None, stream=None):
    ws_ptr, ws_bytes = _ws(workspace)
    rc = _lib.mxc_conv2d_fwd_transform(N, C, H, W, K, R, S, stride, pad, dtype, layout, _ptr(x), _ptr(w), _ptr(bias), int(relu),
                                       _ptr(y), ws_ptr, ws_bytes, _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def mxc_conv2d_prepare_input(N, C, H, W, K, R, S, stride, pad, dtype, layout, x, x_prepared, stream=None):
    rc = _lib.mxc_conv2d_prepare_input(N, C, H, W, K, R, S, stride, pad, dtype, layout, _ptr(x), _ptr(x_prepared),
                                       _nbytes(x_prepared), _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_conv2d_fwd_prepared_input(N, C, H, W, K, R, S, stride, pad, dtype, layout, x_prepared, w, bias, relu, y, workspace=None,
                                  stream=None):
    ws_ptr, ws_bytes = _ws(workspace)
    rc = _lib.mxc_conv2d_fwd_prepared_input(N, C, H, W, K, R, S, stride, pad, dtype, layout, _ptr(x_prepared), _nbytes(x_prepared),
                                            _ptr(w), _ptr(bias), int(relu), _ptr(y), ws_ptr, ws_bytes, _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_conv2d_bwd_weight_prepared_input(N, C, H, W, K, R, S, stride, pad, dtype, layout, x_prepared, dy, dw, dw_dtype,
                                         workspace=None, stream=None):
    ws_ptr, ws_bytes = _ws(workspace)
    rc = _lib.mxc_conv2d_bwd_weight_prepared_input(N, C, H, W, K, R, S, stride, pad, dtype, layout, _ptr(x_prepared),
                                                   _nbytes(x_prepared), _ptr(dy), _ptr(dw), dw_dtype, ws_ptr, ws_bytes,
                                                   _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_bias_grad(N, K, P, Q, dtype, layout, dy, db, workspace=None, stream=None):
    ws_ptr, ws_bytes = _ws(workspace)
    rc = _lib.mxc_bias_grad(N, K, P, Q, dtype, layout, _ptr(dy), _ptr(db), ws_ptr, ws_bytes, _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_fc_fwd(N, C, K, dtype, x, w, bias, relu, y, workspace=None, stream=None):
    ws_ptr, ws_bytes = _ws(workspace)
    rc = _lib.mxc_fc_fwd(N, C, K, dtype, _ptr(x), _ptr(w), _ptr(bias), int(relu), _ptr(y), ws_ptr, ws_bytes, _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_fc_bwd_data(N, C, K, dtype, dy, w, x_mask, dx, workspace=None, stream=None):
    ws_ptr, ws_bytes = _ws(workspace)
    rc = _lib.mxc_fc_bwd_data(N, C, K, dtype, _ptr(dy), _ptr(w), _ptr(x_mask), _ptr(dx), ws_ptr, ws_bytes, _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_fc_bwd_weight(N, C, K, dtype, x, dy, dw, workspace=None, stream=None):
    ws_ptr, ws_bytes = _ws(workspace)
    rc = _lib.mxc_fc_bwd_weight(N, C, K, dtype, _ptr(x), _ptr(dy), _ptr(dw), ws_ptr, ws_bytes, _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_softmax_fwd(N, K, dtype, z, p, stream=None):
    rc = _lib.mxc_softmax_fwd(N, K, dtype, _ptr(z), _ptr(p), _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_softmax_xent_bwd(N, K, dtype, p, labels, scale, dz, stream=None):
    rc = _lib.mxc_softmax_xent_bwd(N, K, dtype, _ptr(p), _ptr(labels), scale, _ptr(dz), _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_sgd_update(w, g, v, w_bf16, lr, momentum, wd, stream=None):
    """In-place update of the fp32 tensors w (and v, may be None); optional bf16 copy of the new w."""
    rc = _lib.mxc_sgd_update(w.numel(), _ptr(w), _ptr(g), _ptr(v), _ptr(w_bf16), lr, momentum, wd, _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_layout_convert(n, c, h, w, dtype, src_layout, dst_layout, src, dst, stream=None):
    rc = _lib.mxc_layout_convert(n, c, h, w, dtype, src_layout, dst_layout, _ptr(src), _ptr(dst), _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)


def mxc_probe_mfma(workgroups, iters, out, stream=None) -> float:
    """Enqueue the matrix-pipe probe; returns the floating-point operations of that launch."""
    flops = ctypes.c_double(0.0)
    rc = _lib.mxc_probe_mfma(workgroups, iters, _ptr(out), out.numel() * out.element_size(), ctypes.byref(flops),
                             _stream(stream))
    if rc != MXC_OK:
        raise MxcError(rc)
    return float(flops.value)


def raw():
    """The ctypes library handle (tests of the error paths pass raw pointers)."""
    return _lib


def alloc_workspace(nbytes: int, device="cuda"):
    """A torch byte tensor of at least nbytes (None when nbytes == 0)."""
    if nbytes == 0:
        return None
    return torch.empty(nbytes, dtype=torch.uint8, device=device)
