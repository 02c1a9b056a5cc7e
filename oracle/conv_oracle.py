"""ctypes front end of oracle/conv_oracle.c.  TEST INFRASTRUCTURE ONLY.

Every function takes float32 numpy arrays in NCHW / KCRS order (the exact values
the GPU path is given: fp32, or bf16 widened to fp32) and returns float64
results computed by the plain loop nests in conv_oracle.c.  Nothing in the
product package imports this module, and this module imports nothing from it.

The operations are the convolution layer's forward pass and its two
derivatives (MXNet paper, Section 2.1 for forward/backward of a symbol and
Section 3.1 for the hand-written "big" layer operators); the paper prints no
formula, so conv_oracle.c's header states the definition used.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libconv_oracle.so")
_lib = None

_I = ctypes.c_int
_LL = ctypes.c_longlong
_FP = ctypes.POINTER(ctypes.c_float)
_DP = ctypes.POINTER(ctypes.c_double)
_LP = ctypes.POINTER(ctypes.c_longlong)


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from oracle.build_oracle import build
        build()
    lib = ctypes.CDLL(_LIB_PATH)
    nine = [_I] * 9
    lib.orc_out_dim.argtypes = [_I, _I, _I, _I]
    lib.orc_out_dim.restype = _I
    for name in ("orc_conv2d_fwd", "orc_conv2d_bwd_data", "orc_conv2d_bwd_weight"):
        f = getattr(lib, name)
        f.argtypes = nine + [_FP, _FP, _DP]
        f.restype = None
    for name in ("orc_conv2d_fwd_at", "orc_conv2d_bwd_data_at", "orc_conv2d_bwd_weight_at"):
        f = getattr(lib, name)
        f.argtypes = nine + [_FP, _FP, _LL, _LP, _DP, _DP]
        f.restype = None
    lib.orc_num_threads.argtypes = []
    lib.orc_num_threads.restype = _I
    _lib = lib
    return lib


def _f32(a, shape):
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _fp(a):
    return a.ctypes.data_as(_FP)


def _dp(a):
    return a.ctypes.data_as(_DP)


def out_dim(size, filt, stride, pad):
    return int(_load().orc_out_dim(size, filt, stride, pad))


def num_threads():
    return int(_load().orc_num_threads())


def _check(N, C, H, W, K, R, S, stride, pad):
    if min(N, C, H, W, K, R, S, stride) <= 0 or pad < 0 or H + 2 * pad < R or W + 2 * pad < S:
        raise ValueError("invalid convolution shape")


def conv2d_fwd(x, w, stride, pad):
    """y[N,K,P,Q] (float64) from x[N,C,H,W], w[K,C,R,S]."""
    N, C, H, W = x.shape
    K, C2, R, S = w.shape
    assert C2 == C
    _check(N, C, H, W, K, R, S, stride, pad)
    x = _f32(x, (N, C, H, W)); w = _f32(w, (K, C, R, S))
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    y = np.empty((N, K, P, Q), dtype=np.float64)
    _load().orc_conv2d_fwd(N, C, H, W, K, R, S, stride, pad, _fp(x), _fp(w), _dp(y))
    return y


def conv2d_bwd_data(dy, w, x_shape, stride, pad):
    """dx[N,C,H,W] (float64) from dy[N,K,P,Q], w[K,C,R,S]."""
    N, C, H, W = x_shape
    K, C2, R, S = w.shape
    assert C2 == C
    _check(N, C, H, W, K, R, S, stride, pad)
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    dy = _f32(dy, (N, K, P, Q)); w = _f32(w, (K, C, R, S))
    dx = np.empty((N, C, H, W), dtype=np.float64)
    _load().orc_conv2d_bwd_data(N, C, H, W, K, R, S, stride, pad, _fp(dy), _fp(w), _dp(dx))
    return dx


def conv2d_bwd_weight(x, dy, w_shape, stride, pad):
    """dw[K,C,R,S] (float64) from x[N,C,H,W], dy[N,K,P,Q]."""
    N, C, H, W = x.shape
    K, C2, R, S = w_shape
    assert C2 == C
    _check(N, C, H, W, K, R, S, stride, pad)
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    x = _f32(x, (N, C, H, W)); dy = _f32(dy, (N, K, P, Q))
    dw = np.empty((K, C, R, S), dtype=np.float64)
    _load().orc_conv2d_bwd_weight(N, C, H, W, K, R, S, stride, pad, _fp(x), _fp(dy), _dp(dw))
    return dw


def _at(name, dims, a, b, idx):
    idx = np.ascontiguousarray(idx, dtype=np.int64).ravel()
    val = np.empty(idx.size, dtype=np.float64)
    den = np.empty(idx.size, dtype=np.float64)
    getattr(_load(), name)(*dims, _fp(a), _fp(b), idx.size,
                           idx.ctypes.data_as(_LP), _dp(val), _dp(den))
    return val, den


def conv2d_fwd_at(x, w, stride, pad, idx):
    """(value, D) of y at flat NKPQ indices idx; D = sum |x||w| over the same taps."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    _check(N, C, H, W, K, R, S, stride, pad)
    x = _f32(x, (N, C, H, W)); w = _f32(w, (K, C, R, S))
    return _at("orc_conv2d_fwd_at", (N, C, H, W, K, R, S, stride, pad), x, w, idx)


def conv2d_bwd_data_at(dy, w, x_shape, stride, pad, idx):
    """(value, D) of dx at flat NCHW indices idx; D = sum |dy||w|."""
    N, C, H, W = x_shape
    K, _, R, S = w.shape
    _check(N, C, H, W, K, R, S, stride, pad)
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    dy = _f32(dy, (N, K, P, Q)); w = _f32(w, (K, C, R, S))
    return _at("orc_conv2d_bwd_data_at", (N, C, H, W, K, R, S, stride, pad), dy, w, idx)


def conv2d_bwd_weight_at(x, dy, w_shape, stride, pad, idx):
    """(value, D) of dw at flat KCRS indices idx; D = sum |dy||x|."""
    N, C, H, W = x.shape
    K, _, R, S = w_shape
    _check(N, C, H, W, K, R, S, stride, pad)
    P, Q = out_dim(H, R, stride, pad), out_dim(W, S, stride, pad)
    x = _f32(x, (N, C, H, W)); dy = _f32(dy, (N, K, P, Q))
    return _at("orc_conv2d_bwd_weight_at", (N, C, H, W, K, R, S, stride, pad), x, dy, idx)


# ---- convolution grouped with its neighbours (bias, ReLU) -----------------------------------
# The paper groups operators into a single call where it can (Section 3.1, graph optimisation) and
# builds networks as layer => Activation(relu) => layer (Section 2.1, symbol construction).  These
# are the plain definitions of the grouped forms, built from the loop nests above with elementwise
# numpy steps in float64; nothing is blocked or reordered.

def conv2d_fwd_bias_act(x, w, bias, relu, stride, pad):
    """a = act(conv(x, w) + bias[k]), act = max(0, .) when relu else identity.  Returns (a, D) with
    D = sum |x||w| + |bias|, the magnitude the error metric divides by."""
    bias = np.asarray(bias, dtype=np.float64)
    K = np.asarray(w).shape[0]
    if bias.shape != (K,):
        raise ValueError("bias must have one entry per output channel")
    z = conv2d_fwd(x, w, stride, pad) + bias[None, :, None, None]
    den = conv2d_fwd(np.abs(x), np.abs(w), stride, pad) + np.abs(bias)[None, :, None, None]
    return (np.maximum(z, 0.0) if relu else z), den


def conv2d_bwd_data_relu(dy, w, x, stride, pad):
    """Gradient with respect to the pre-activation that produced x = max(0, z):
    dz = conv^T(dy, w) where x > 0, else 0 (the derivative of max(0, .) is taken as 0 at 0).
    Returns (dz, D) with D = sum |dy||w| where x > 0, else 0."""
    x = np.asarray(x)
    g = conv2d_bwd_data(dy, w, x.shape, stride, pad)
    den = conv2d_bwd_data(np.abs(dy), np.abs(w), x.shape, stride, pad)
    keep = x > 0
    return np.where(keep, g, 0.0), np.where(keep, den, 0.0)


def bias_grad(dy):
    """db[k] = sum over images and pixels of dy[n, k, p, q] (the derivative of z + bias[k] summed
    over everything the bias is added to).  Returns (db, D) with D = sum |dy|."""
    dy = np.asarray(dy, dtype=np.float64)
    if dy.ndim != 4:
        raise ValueError("dy must be N,K,P,Q")
    return dy.sum(axis=(0, 2, 3)), np.abs(dy).sum(axis=(0, 2, 3))


# ---- the weight update that consumes dw ------------------------------------------------------
# The paper writes the update as w = w - eta*g (Section 2.2) and trains with learning rate .05,
# momentum .9 and weight decay 1e-4 (Section 4) without printing the momentum form; the reading
# taken here is the classic one:  v' = mu*v - eta*(g + lambda*w),  w' = w + v'.

def sgd_update(w, g, v, lr, momentum, wd):
    """One update in float64.  Returns (w', v')."""
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    v = np.zeros_like(w) if v is None else np.asarray(v, dtype=np.float64)
    v2 = momentum * v - lr * (g + wd * w)
    return w + v2, v2


# ---- FullyConnected (the layer of the paper's running example, Section 2.1) ---------------------
# y[n, k] = sum_c x[n, c] * w[k, c] (+ bias[k], optional ReLU) and its derivatives, written as the
# matrix products they are, in float64.  Each returns (value, D) with D the sum of |a||b| of the
# same terms (plus |bias| forward).

def fc_fwd(x, w, bias=None, relu=False):
    x = np.asarray(x, dtype=np.float64); w = np.asarray(w, dtype=np.float64)
    if x.ndim != 2 or w.ndim != 2 or x.shape[1] != w.shape[1]:
        raise ValueError("x must be [N, C], w [K, C]")
    z = x @ w.T
    den = np.abs(x) @ np.abs(w).T
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64)
        z = z + b[None, :]
        den = den + np.abs(b)[None, :]
    return (np.maximum(z, 0.0) if relu else z), den


def fc_bwd_data(dy, w, x_mask=None):
    """dx = dy @ w; with x_mask (the layer's input, a ReLU output) dx is 0 where x_mask <= 0."""
    dy = np.asarray(dy, dtype=np.float64); w = np.asarray(w, dtype=np.float64)
    g = dy @ w
    den = np.abs(dy) @ np.abs(w)
    if x_mask is not None:
        keep = np.asarray(x_mask) > 0
        g = np.where(keep, g, 0.0); den = np.where(keep, den, 0.0)
    return g, den


def fc_bwd_weight(x, dy):
    """dw[k, c] = sum_n dy[n, k] * x[n, c]."""
    x = np.asarray(x, dtype=np.float64); dy = np.asarray(dy, dtype=np.float64)
    return dy.T @ x, np.abs(dy).T @ np.abs(x)


# ---- Softmax output layer (the last layer of the paper's running example, Section 2.1) ---------------
# Forward: p[n, k] = exp(z[n, k]) / sum_j exp(z[n, j]).  As an output (loss) layer its gradient with
# respect to z for the cross-entropy against integer labels is (p - onehot(label)) * scale.

def softmax_fwd(z):
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def softmax_xent_bwd(p, labels, scale=1.0):
    p = np.asarray(p, dtype=np.float64)
    g = p.copy()
    g[np.arange(p.shape[0]), np.asarray(labels, dtype=np.int64)] -= 1.0
    return g * scale
