"""Helpers for the GPU parity tests: moving seeded numpy inputs onto the GPU in the
layout/dtype an entry point wants, calling the C ABI through the binding, and the
error metric.  No convolution arithmetic lives here."""
import numpy as np
import torch

from paper_1512_01274_amd import inputs as gen

# Tolerances of the error metric  max |gpu - oracle| / D,  D = sum |a||b| over the taps of that output.
TOL = {"f32": 1e-5, "bf16": 1e-2}


to_device = gen.to_device
to_host_f64 = gen.to_host_f64


def nchw_to_nhwc(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a.transpose(0, 2, 3, 1))


def nhwc_to_nchw(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a.transpose(0, 3, 1, 2))


class Runner:
    """Calls the three entry points for one problem; inputs are NCHW/KCRS float32 numpy arrays."""

    def __init__(self, mxc, dims, dtype: str, layout: str):
        self.mxc, self.dims, self.dtype, self.layout = mxc, tuple(dims), dtype, layout
        self.N, self.C, self.H, self.W, self.K, self.R, self.S, self.stride, self.pad = self.dims
        self.P = (self.H + 2 * self.pad - self.R) // self.stride + 1
        self.Q = (self.W + 2 * self.pad - self.S) // self.stride + 1
        self.dt = mxc.MXC_BF16 if dtype == "bf16" else mxc.MXC_F32
        self.lay = mxc.MXC_NHWC if layout == "nhwc" else mxc.MXC_NCHW
        self.tdtype = torch.bfloat16 if dtype == "bf16" else torch.float32

    def _in(self, a):
        return to_device(nchw_to_nhwc(a) if self.layout == "nhwc" else a, self.dtype)

    def _out(self, t, shape_nchw):
        n, c, h, w = shape_nchw
        a = to_host_f64(t)
        if self.layout == "nhwc":
            return nhwc_to_nchw(a.reshape(n, h, w, c))
        return a.reshape(n, c, h, w)

    def _ws(self, op):
        nbytes = self.mxc.mxc_conv2d_workspace_bytes(op, *self.dims, self.dt, self.lay)
        return self.mxc.alloc_workspace(nbytes)

    def fwd(self, x, w, return_tensor=False):
        y = torch.full((self.N * self.K * self.P * self.Q,), float("nan"), dtype=self.tdtype, device="cuda")
        self.mxc.mxc_conv2d_fwd(*self.dims, self.dt, self.lay, self._in(x), self._in(w), y, self._ws(self.mxc.MXC_FWD))
        torch.cuda.synchronize()
        return y if return_tensor else self._out(y, (self.N, self.K, self.P, self.Q))

    def bwd_data(self, dy, w, return_tensor=False):
        dx = torch.full((self.N * self.C * self.H * self.W,), float("nan"), dtype=self.tdtype, device="cuda")
        self.mxc.mxc_conv2d_bwd_data(*self.dims, self.dt, self.lay, self._in(dy), self._in(w), dx,
                                     self._ws(self.mxc.MXC_BWD_DATA))
        torch.cuda.synchronize()
        return dx if return_tensor else self._out(dx, (self.N, self.C, self.H, self.W))

    def bwd_weight(self, x, dy, return_tensor=False):
        dw = torch.full((self.K * self.C * self.R * self.S,), float("nan"), dtype=torch.float32, device="cuda")
        self.mxc.mxc_conv2d_bwd_weight(*self.dims, self.dt, self.lay, self._in(x), self._in(dy), dw,
                                       self._ws(self.mxc.MXC_BWD_WEIGHT))
        torch.cuda.synchronize()
        if return_tensor:
            return dw
        a = dw.cpu().numpy().astype(np.float64)
        if self.layout == "nhwc":
            return nhwc_to_nchw(a.reshape(self.K, self.R, self.S, self.C))
        return a.reshape(self.K, self.C, self.R, self.S)


def metric(gpu: np.ndarray, ref: np.ndarray, den: np.ndarray) -> float:
    """max over outputs of |gpu-ref|/D; where D == 0 the GPU value must be exactly 0 (returns inf if not)."""
    gpu, ref, den = gpu.ravel(), ref.ravel(), den.ravel()
    if not np.isfinite(gpu).all():
        return float("inf")
    zero = den == 0
    if zero.any() and (gpu[zero] != 0).any():
        return float("inf")
    if zero.all():
        return 0.0
    return float((np.abs(gpu[~zero] - ref[~zero]) / den[~zero]).max())


def tight_bound(ref: np.ndarray, den: np.ndarray, dtype: str, out_is_bf16: bool) -> np.ndarray:
    """Per-output absolute error allowed by the arithmetic itself (much tighter than TOL):
    fp32 accumulation error  c * 2^-24 * D  (c covers sums of a few thousand terms in any order)
    plus, for bf16 outputs, half an ulp of the result (2^-9 relative, 2^-8 used)."""
    b = 64 * 2.0 ** -24 * den
    if out_is_bf16:
        b = b + 2.0 ** -8 * np.abs(ref)
    return b + 1e-30


def transform_domain_budget(x: np.ndarray, w: np.ndarray, pad: int) -> np.ndarray:
    """Worst-case effect of the two bf16 roundings of the transform-domain 3x3 forward (2x2 output blocks from 4x4
    patches), per output element: W[n,k,p,q] = (|At| (sum_c |G g Gt| * |Bt d B|) |A|), the quantity its error bound
    multiplies by 2^-8.  x is NCHW, w is KCRS, float64 arithmetic."""
    G = np.array([[1, 0, 0], [.5, .5, .5], [.5, -.5, .5], [0, 0, 1]], dtype=np.float64)
    Bt = np.array([[1, 0, -1, 0], [0, 1, 1, 0], [0, -1, 1, 0], [0, 1, 0, -1]], dtype=np.float64)
    At = np.array([[1, 1, 1, 0], [0, 1, -1, -1]], dtype=np.float64)
    N, C, H, W_ = x.shape
    K = w.shape[0]
    P, Q = H + 2 * pad - 2, W_ + 2 * pad - 2
    TP, TQ = (P + 1) // 2, (Q + 1) // 2
    xp = np.zeros((N, C, 2 * TP + 2, 2 * TQ + 2), dtype=np.float64)
    hh, ww = min(H, xp.shape[2] - pad), min(W_, xp.shape[3] - pad)
    xp[:, :, pad:pad + hh, pad:pad + ww] = x[:, :, :hh, :ww]
    U = np.abs(np.einsum("ir,kcrs,js->kcij", G, w.astype(np.float64), G))
    out = np.zeros((N, K, 2 * TP, 2 * TQ), dtype=np.float64)
    aAt = np.abs(At)
    for tp in range(TP):
        for tq in range(TQ):
            d = xp[:, :, 2 * tp:2 * tp + 4, 2 * tq:2 * tq + 4]
            V = np.abs(np.einsum("ia,ncab,jb->ncij", Bt, d, Bt))
            Wm = np.einsum("kcij,ncij->nkij", U, V)
            out[:, :, 2 * tp:2 * tp + 2, 2 * tq:2 * tq + 2] = np.einsum("ai,nkij,bj->nkab", aAt, Wm, aAt)
    return out[:, :, :P, :Q]
