/*
 * mxc.h -- C ABI of the MI355X (gfx950) conv2d library.
 *
 * The three compute calls are the convolution layer of the MXNet paper: the
 * hand-optimised "big" operator of Section 3.1 (Graph Optimization), whose
 * forward and backward evaluation Section 2.1 describes and whose kernels
 * Section 4 ("Raw performance") reports as taking most of the run time of the
 * CNN benchmarks.  The paper prints no formula; the definitions below are the
 * ones this library implements.
 *
 * Notation.  x[N,C,H,W] input, w[K,C,R,S] filter, y/dy[N,K,P,Q] output and its
 * gradient, with
 *     P = floor((H + 2*pad - R)/stride) + 1,  Q = floor((W + 2*pad - S)/stride) + 1.
 * One stride and one pad serve both axes; dilation 1, groups 1, no bias in the three plain calls;
 * cross-correlation (no filter flip); x outside the image reads as 0.
 *
 * Common rules for every call.
 *   - All data pointers are DEVICE pointers on the current HIP device, 16-byte
 *     aligned, owned by the caller; the library allocates no device memory,
 *     never synchronises and never changes the current device.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  Calls return as soon as the launches are queued.
 *   - `dtype` is the element type of x, w, y, dy, dx: MXC_F32, or MXC_BF16
 *     (bf16 storage, fp32 accumulation, results rounded to nearest-even).
 *     dw is fp32 for both dtypes (mxc_conv2d_bwd_weight_bf16 and the prepared-input
 *     form with dw_dtype MXC_BF16 round that fp32 sum once to bf16).
 *   - `layout` says how the caller's tensors are stored:
 *       MXC_NCHW: x[N][C][H][W], w/dw[K][C][R][S], y/dy[N][K][P][Q]
 *       MXC_NHWC: x[N][H][W][C], w/dw[K][R][S][C], y/dy[N][P][Q][K]
 *     all dense.  Kernels work in NHWC/KRSC; NCHW tensors are converted through
 *     the workspace.
 *   - Outputs are fully overwritten (no accumulation into them).
 *   - `workspace` is scratch memory of at least the size reported by
 *     mxc_conv2d_workspace_bytes for the same arguments (may be NULL when that
 *     size is 0).  Its contents are undefined afterwards.  Two calls that share
 *     a workspace must be ordered on one stream.
 *   - Return value: MXC_OK or an error code.  Argument errors (every code but
 *     MXC_ERR_LAUNCH) are found before anything is launched; after MXC_ERR_LAUNCH
 *     some of the call's kernels may already be queued and the output is undefined.
 *     No call throws, aborts or exits.  Shapes are checked before pointers.
 */
#ifndef MXC_H
#define MXC_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MXC_OK = 0,
    MXC_ERR_NULL = 1,        /* a required pointer is NULL                         */
    MXC_ERR_SHAPE = 2,       /* non-positive dim/stride, negative pad, empty output */
    MXC_ERR_UNSUPPORTED = 3, /* unknown dtype / layout / pass                       */
    MXC_ERR_WORKSPACE = 4,   /* workspace missing or smaller than required          */
    MXC_ERR_ALIGN = 5,       /* a pointer is not 16-byte aligned                    */
    MXC_ERR_LAUNCH = 6       /* the HIP runtime rejected a kernel launch            */
};

enum { MXC_F32 = 0, MXC_BF16 = 1 };
enum { MXC_NCHW = 0, MXC_NHWC = 1 };
enum { MXC_FWD = 0, MXC_BWD_DATA = 1, MXC_BWD_WEIGHT = 2,
       /* the following: mxc_conv2d_workspace_bytes only */
       MXC_BWD_DATA_RELU = 3, MXC_BIAS_GRAD = 4,
       MXC_BWD_DATA_FILTER = 5,          /* bytes of the prepared filter of mxc_conv2d_bwd_data_prepare_filter */
       MXC_BWD_DATA_PREPARED = 6,        /* workspace of mxc_conv2d_bwd_data_prepared without x_mask           */
       MXC_BWD_DATA_PREPARED_RELU = 7,   /* ... with x_mask                                                     */
       MXC_BWD_WEIGHT_BF16 = 8,          /* workspace of mxc_conv2d_bwd_weight_bf16                             */
       MXC_INPUT_PREPARED = 9,           /* bytes of the prepared input of mxc_conv2d_prepare_input (0: none)   */
       MXC_FWD_PREPARED_INPUT = 10,      /* workspace of mxc_conv2d_fwd_prepared_input                          */
       MXC_BWD_WEIGHT_PREPARED_INPUT = 11,       /* workspace of mxc_conv2d_bwd_weight_prepared_input, fp32 dw  */
       MXC_BWD_WEIGHT_PREPARED_INPUT_BF16 = 12,  /* ... bf16 dw                                                 */
       MXC_FWD_TRANSFORM = 13 };         /* workspace of mxc_conv2d_fwd_transform                               */

/*
 * Forward (the layer's "forward" evaluation, paper Section 2.1):
 *   y[n,k,p,q] = sum_{c,r,s} x[n,c,p*stride-pad+r,q*stride-pad+s] * w[k,c,r,s]
 * x, w: inputs; y: output (N*K*P*Q elements of `dtype`).
 */
int mxc_conv2d_fwd(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                   int dtype, int layout,
                   const void *x, const void *w, void *y,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward w.r.t. the input (derivative of forward in x; paper Section 2.1,
 * "backward"):
 *   dx[n,c,h,v] = sum over (k,r,s) such that p=(h+pad-r)/stride and
 *                 q=(v+pad-s)/stride are integers inside the output,
 *                 of dy[n,k,p,q] * w[k,c,r,s].
 * Every element of dx is written; positions no filter tap reaches get 0.
 * dy, w: inputs; dx: output (N*C*H*W elements of `dtype`).
 */
int mxc_conv2d_bwd_data(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                        int dtype, int layout,
                        const void *dy, const void *w, void *dx,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward w.r.t. the filter (derivative of forward in w; the gradient that the
 * paper's update step w -= eta*g of Section 2.2 consumes):
 *   dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*stride-pad+r,q*stride-pad+s]
 * x, dy: inputs of `dtype`; dw: output, K*C*R*S fp32 values in the filter order
 * of `layout`.  The reduction is split across workgroups and summed in a fixed
 * order: results are bit-identical from run to run.
 */
int mxc_conv2d_bwd_weight(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                          int dtype, int layout,
                          const void *x, const void *dy, void *dw,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward w.r.t. the filter with the gradient delivered in bf16: the same sums as mxc_conv2d_bwd_weight
 * (fp32 accumulation, fp32 split partial sums added in a fixed order), rounded ONCE to bf16 (nearest even) by
 * the kernel that forms the final sum - for a gradient exchange or an optimizer that takes bf16 (half the bytes
 * of the push of paper Section 2.3).  dtype must be MXC_BF16 (else MXC_ERR_UNSUPPORTED); dw: K*C*R*S bf16
 * values in the filter order of `layout`.  Workspace: query MXC_BWD_WEIGHT_BF16.  Otherwise as
 * mxc_conv2d_bwd_weight.
 */
int mxc_conv2d_bwd_weight_bf16(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               int dtype, int layout,
                               const void *x, const void *dy, void *dw,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * mxc_conv2d_bwd_weight for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * computation, kernels and results as mxc_conv2d_bwd_weight, with the split-reduction partial sums
 * (and, for MXC_NCHW, the converted operands) held in a 64 MiB array that is part of the library's
 * device code - one copy per GPU, kept until the process ends.  The call allocates nothing.  x, dy,
 * dw as in mxc_conv2d_bwd_weight, still caller-owned.
 *   - Problems whose scratch need (what mxc_conv2d_workspace_bytes reports for MXC_BWD_WEIGHT)
 *     exceeds 64 MiB are rejected with MXC_ERR_WORKSPACE before anything is launched.
 *   - All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different
 *     streams, or several host threads) race on it; order them on one stream.  The array keeps the
 *     last call's contents; no call depends on them.
 *   - The first call on a device looks up the array's device address (hipGetSymbolAddress): make
 *     that call outside any stream capture.  If the lookup fails: MXC_ERR_LAUNCH, nothing launched.
 * Other errors as mxc_conv2d_bwd_weight.
 */
int mxc_conv2d_bwd_weight_static(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                 int dtype, int layout,
                                 const void *x, const void *dy, void *dw, void *hip_stream);

/*
 * Convolution grouped with the operations that follow it (the paper groups operators into a
 * single call where it can, Section 3.1 "Graph Optimization", and chains layers as
 * layer => Activation(relu) => layer, Section 2.1):
 *   y[n,k,p,q] = act( forward(x, w)[n,k,p,q] + bias[k] ),   act(t) = max(0, t) if relu == 1, t if relu == 0.
 * bias: K fp32 values in device memory (4-byte aligned), or NULL for no bias.  The sum is formed
 * in fp32 and rounded once to `dtype`.  Everything else (layouts, workspace = that of MXC_FWD,
 * ownership, errors) as mxc_conv2d_fwd; relu outside {0,1}: MXC_ERR_UNSUPPORTED.
 */
int mxc_conv2d_fwd_bias_act(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                            int dtype, int layout,
                            const void *x, const void *w, const float *bias, int relu, void *y,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward w.r.t. the input, grouped with the derivative of the ReLU that produced the input:
 * with x = max(0, z) the output of the layer below,
 *   dz[n,c,h,v] = backward_data(dy, w)[n,c,h,v]  if x[n,c,h,v] > 0,  else 0
 * (the derivative of max(0, .) at 0 is taken as 0).  x: N*C*H*W elements of `dtype` in `layout`
 * (read only); dz is written to dx.  Workspace: query with pass MXC_BWD_DATA_RELU.  Otherwise as
 * mxc_conv2d_bwd_data.
 */
int mxc_conv2d_bwd_data_relu(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                             int dtype, int layout,
                             const void *dy, const void *w, const void *x, void *dx,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward w.r.t. the input with the filter prepared ahead of time.  Every backward-data path first brings
 * the filter into the form its kernels read (re-packed per stride residue class, transposed, ...): work that
 * depends on w alone.  A training loop changes w once per step (the update of Section 2.2), serving never:
 *   mxc_conv2d_bwd_data_prepare_filter  writes that form of w into w_prepared (device memory of the caller, at
 *       least mxc_conv2d_workspace_bytes(MXC_BWD_DATA_FILTER, ...) bytes, 16-byte aligned; opaque contents, valid
 *       for exactly these N..pad, dtype and layout until w changes);
 *   mxc_conv2d_bwd_data_prepared        is mxc_conv2d_bwd_data (x_mask == NULL) or mxc_conv2d_bwd_data_relu
 *       (x_mask = the layer's input) reading w_prepared instead of w; same results bit for bit.  Workspace:
 *       query MXC_BWD_DATA_PREPARED / MXC_BWD_DATA_PREPARED_RELU.
 * prepared_bytes: size of the w_prepared buffer (checked against the required size: MXC_ERR_WORKSPACE).
 * Everything else as mxc_conv2d_bwd_data.
 */
int mxc_conv2d_bwd_data_prepare_filter(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                       int dtype, int layout,
                                       const void *w, void *w_prepared, size_t prepared_bytes, void *hip_stream);
int mxc_conv2d_bwd_data_prepared(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                 int dtype, int layout,
                                 const void *dy, const void *w_prepared, size_t prepared_bytes, const void *x_mask, void *dx,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Forward and backward-weight on an input prepared once.  Layers whose channel count is not a multiple of 8
 * (the first layer of every network of Section 4: C = 3) first bring x into the form their kernels read -
 * space-to-depth packed for strided filters, zero-bordered with 4 channels per pixel, or channel-padded -
 * and both passes of a training step (Section 2.1: forward, then the gradient of the weights) read the same
 * form of the same x:
 *   mxc_conv2d_prepare_input             writes that form into x_prepared (device memory of the caller, at least
 *       mxc_conv2d_workspace_bytes(MXC_INPUT_PREPARED, ...) bytes, 16-byte aligned; opaque contents, valid for
 *       exactly these N..pad, dtype and layout until x changes).  A layer that reads x as it is has 0 bytes:
 *       the call does nothing (x_prepared may be NULL) and the two calls below take x itself as x_prepared;
 *   mxc_conv2d_fwd_prepared_input        is mxc_conv2d_fwd_bias_act (bias may be NULL, relu 0 or 1) reading
 *       x_prepared; same results bit for bit.  Workspace: query MXC_FWD_PREPARED_INPUT;
 *   mxc_conv2d_bwd_weight_prepared_input is mxc_conv2d_bwd_weight (dw_dtype MXC_F32) or mxc_conv2d_bwd_weight_bf16
 *       (dw_dtype MXC_BF16) reading x_prepared; same results bit for bit.  Workspace: query
 *       MXC_BWD_WEIGHT_PREPARED_INPUT / MXC_BWD_WEIGHT_PREPARED_INPUT_BF16.
 * layout must be MXC_NHWC (MXC_ERR_UNSUPPORTED otherwise: the NCHW boundary converts every operand per call).
 * prepared_bytes: size of the x_prepared buffer (checked: MXC_ERR_WORKSPACE).  Everything else as the calls named.
 */
int mxc_conv2d_prepare_input(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                             int dtype, int layout,
                             const void *x, void *x_prepared, size_t prepared_bytes, void *hip_stream);
int mxc_conv2d_fwd_prepared_input(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                  int dtype, int layout,
                                  const void *x_prepared, size_t prepared_bytes, const void *w, const float *bias, int relu,
                                  void *y, void *workspace, size_t workspace_bytes, void *hip_stream);
int mxc_conv2d_bwd_weight_prepared_input(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                                         int dtype, int layout,
                                         const void *x_prepared, size_t prepared_bytes, const void *dy, void *dw, int dw_dtype,
                                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Forward by another algorithm: the 3x3 stride-1 convolution evaluated in a transform domain (minimal filtering,
 * 2x2 output blocks from 4x4 input patches: 16 multiplications per channel and block instead of 36), the same
 * y = act(conv(x, w) + bias) as mxc_conv2d_fwd_bias_act (Section 2.1; one of the hand-optimised "big" operators
 * of Section 3.1).  Filter and input are transformed, rounded once to bf16 and multiplied on the matrix cores as
 * 16 independent GEMMs with fp32 sums; the result is transformed back and rounded once.  Its error is therefore
 * not that of the direct form: |y - exact| <= 2^-8 * W + 2^-8 * |exact|, W = the sum, over the transform-domain
 * entries a result combines, of sum_c |U||V| (U, V the transformed filter and input); for the layers of the
 * benchmark stacks that is well inside 1e-2 of sum |x||w|.
 * Only R = S = 3, stride = 1, dtype MXC_BF16, layout MXC_NHWC, C % 8 == 0 and K % 8 == 0 (MXC_ERR_UNSUPPORTED
 * otherwise; callers fall back to mxc_conv2d_fwd_bias_act).  bias may be NULL, relu is 0 or 1.  Workspace: query
 * MXC_FWD_TRANSFORM (16 transformed copies of the tiled input in bf16 and of the output in fp32: large).
 * Everything else as mxc_conv2d_fwd.
 */
int mxc_conv2d_fwd_transform(int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                             int dtype, int layout,
                             const void *x, const void *w, const float *bias, int relu, void *y,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Gradient of the bias of mxc_conv2d_fwd_bias_act (derivative of forward + bias[k] in bias):
 *   db[k] = sum_{n,p,q} dy[n,k,p,q]
 * dy: N*K*P*Q elements of `dtype` in `layout` (NCHW: [N][K][P][Q]; NHWC: [N][P][Q][K]); db: K fp32
 * values.  Summed in a fixed order (bit-identical from run to run).  Workspace: query
 * mxc_conv2d_workspace_bytes with pass MXC_BIAS_GRAD (only N, K, P, Q matter: pass the layer's
 * shape).  Errors: MXC_ERR_SHAPE, MXC_ERR_UNSUPPORTED, MXC_ERR_NULL, MXC_ERR_ALIGN,
 * MXC_ERR_WORKSPACE, MXC_ERR_LAUNCH.
 */
int mxc_bias_grad(int N, int K, int P, int Q, int dtype, int layout,
                  const void *dy, float *db,
                  void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * FullyConnected (the layer of the paper's running example, Section 2.1), run through the same
 * matrix-core GEMM as the convolutions: it is the convolution with H = W = R = S = 1, for which NCHW
 * and NHWC coincide.  x: [N][C], w: [K][C], y / dy: [N][K], all of `dtype`; dw: [K][C] fp32.
 *   forward:         y[n,k]  = act( sum_c x[n,c] * w[k,c] + bias[k] )     (bias may be NULL; relu 0 or 1)
 *   backward-data:   dx[n,c] = sum_k dy[n,k] * w[k,c],  set to 0 where x_mask[n,c] <= 0 if x_mask != NULL
 *                    (x_mask: the layer's input when that is a ReLU output)
 *   backward-weight: dw[k,c] = sum_n dy[n,k] * x[n,c]
 * Problems of a few hundred rows split their long reduction over workgroups (fp32 partial sums added
 * in a fixed order: deterministic).  Workspace: mxc_conv2d_workspace_bytes(pass, N, C, 1, 1, K, 1, 1,
 * 1, 0, dtype, MXC_NHWC, ...) with pass MXC_FWD, MXC_BWD_DATA_RELU (with or without mask) or
 * MXC_BWD_WEIGHT.  Ownership, stream and error behaviour as the convolution entry points.
 */
int mxc_fc_fwd(int N, int C, int K, int dtype, const void *x, const void *w, const float *bias, int relu, void *y,
               void *workspace, size_t workspace_bytes, void *hip_stream);
int mxc_fc_bwd_data(int N, int C, int K, int dtype, const void *dy, const void *w, const void *x_mask, void *dx,
                    void *workspace, size_t workspace_bytes, void *hip_stream);
int mxc_fc_bwd_weight(int N, int C, int K, int dtype, const void *x, const void *dy, void *dw,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Softmax output layer (the last layer of the paper's running example, Section 2.1).
 *   forward:   p[n,k] = exp(z[n,k] - max_j z[n,j]) / sum_j exp(z[n,j] - max_j z[n,j])      z, p: [N][K] of `dtype`
 *   backward:  dz[n,k] = (p[n,k] - (k == labels[n])) * scale        the gradient of the cross-entropy against integer
 *              labels (device int32, values in [0, K); a value outside selects no class), times `scale` (e.g. 1/N)
 * Arithmetic in fp32, one rounding to `dtype`.  No workspace.  Errors: MXC_ERR_SHAPE, MXC_ERR_UNSUPPORTED,
 * MXC_ERR_NULL, MXC_ERR_ALIGN (16 bytes for tensors, 4 for labels), MXC_ERR_LAUNCH.
 */
int mxc_softmax_fwd(int N, int K, int dtype, const void *z, void *p, void *hip_stream);
int mxc_softmax_xent_bwd(int N, int K, int dtype, const void *p, const int *labels, float scale, void *dz, void *hip_stream);

/*
 * The weight update that consumes dw (the paper's  w = w - eta*g  of Section 2.2, with the
 * momentum and weight decay of its Section 4 experiment; the paper does not print the momentum
 * form, the classic one is used):
 *   v'[i] = momentum*v[i] - lr*(g[i] + wd*w[i]),   w'[i] = w[i] + v'[i],   i < n
 * w: fp32 master weights, updated in place; g: fp32 gradient (mxc_conv2d_bwd_weight's dw, same
 * element order as w); v: fp32 velocity, updated in place, or NULL when momentum == 0 (then
 * v = 0 is used and nothing is stored); w_bf16: if not NULL, receives w' rounded to bf16 (nearest
 * even) for the next forward pass.  All device pointers, 16-byte aligned, caller-owned; n > 0.
 * Errors: MXC_ERR_SHAPE (n == 0 or too large for one launch), MXC_ERR_NULL (w or g NULL, or v NULL
 * with momentum != 0), MXC_ERR_ALIGN, MXC_ERR_LAUNCH.
 */
int mxc_sgd_update(size_t n, float *w, const float *g, float *v, void *w_bf16,
                   float lr, float momentum, float wd, void *hip_stream);

/*
 * Workspace size in bytes that `pass` (MXC_FWD / MXC_BWD_DATA / MXC_BWD_WEIGHT)
 * needs for these arguments, written to *out_bytes (a HOST pointer).  Touches
 * no GPU state.
 */
int mxc_conv2d_workspace_bytes(int pass, int N, int C, int H, int W, int K, int R, int S,
                               int stride, int pad, int dtype, int layout, size_t *out_bytes);

/*
 * Layout conversion of a dense 4-D tensor between [n][c][h][w] and [n][h][w][c]
 * (the conversion a network does once at entry and exit when activations stay
 * NHWC between layers).  Also converts filters KCRS <-> KRSC with n=K, h=R, w=S.
 * src and dst are device pointers and must not overlap.  src_layout ==
 * dst_layout is a plain copy.
 */
int mxc_layout_convert(int n, int c, int h, int w, int dtype, int src_layout, int dst_layout,
                       const void *src, void *dst, void *hip_stream);

/* Static, NUL-terminated description of a status code (host memory, never freed). */
const char *mxc_status_string(int status);

/* Name of the kernel variant the calling thread's last successful compute call
 * chose (for logs and the bench); "" before any call.  Host memory, thread-local. */
const char *mxc_last_variant(void);

/* Library version as major*10000 + minor*100 + patch. */
int mxc_version(void);

/* Tuning aid: name of the index-th tile shape the matrix-core kernels are built in (family 0: forward /
 * backward-data implicit GEMM, family 1: backward-weight, family 2: the whole-launch implicit GEMMs - "igemm_stream"
 * for short reductions and "igemm_window" for multi-tap stride-1 layers of at most 64 channels, each one plan that
 * runs only where its filter tile fits on chip), NULL past the last.  These are the names that
 * mxc_last_variant() reports and that the tuning hooks MXC_FORCE_VARIANT=<name>[+<name of the shape for the
 * rows the last whole round leaves>] and MXC_FORCE_WGRAD=<name>[/<splits>] (environment, read per call) accept;
 * the tuning script and the tests walk the list.  Static host memory. */
const char *mxc_tile_name(int family, int index);

/* Tuning aid: the implicit GEMM (rows M, output columns Co, reduction length Kd) that the calling thread's last
 * forward or backward-data call planned - for first layers that is the GEMM on the packed operands, whose
 * dimensions the caller does not otherwise see.  The tuning script keys its table of measured plans on it.
 * All three are 0 before any such call.  Host only. */
void mxc_last_plan_key(long long *M, int *Co, int *Kd);

/* Measurement aid (not part of the convolution path): enqueues one launch of a
 * register-resident loop of bf16 matrix instructions (v_mfma_f32_32x32x16_bf16, fp32
 * accumulate, no memory traffic) on `workgroups` workgroups of 256 threads, `iters`
 * iterations of four instructions per wave, and stores in *flops (host memory) the number
 * of floating-point operations that launch performs.  The caller times the launch; flops
 * over time is the matrix-pipe ceiling of this device at its sustained clock, the
 * "measured peak" that the benchmark reports beside the published one (the paper, Section 4,
 * compares on measured speed only).  `out`: device buffer of at least workgroups*256 floats
 * (16-byte aligned; receives values of no interest), caller-owned.  Errors: MXC_ERR_NULL,
 * MXC_ERR_SHAPE (non-positive counts), MXC_ERR_WORKSPACE (out too small), MXC_ERR_ALIGN,
 * MXC_ERR_LAUNCH. */
int mxc_probe_mfma(int workgroups, int iters, void *out, size_t out_bytes, double *flops, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MXC_H */
