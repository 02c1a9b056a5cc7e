/*
 * conv_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, double-precision CPU definition of 2-D convolution forward,
 * backward-data and backward-weight.  It exists so that the GPU library can be
 * checked against something written independently of it; only the tests, the
 * smoke check and the bench's cpu_baseline leg may call it.  Nothing here is
 * shared with the GPU path.
 *
 * What it follows.  The MXNet paper names the convolution layer as one of its
 * hand-optimised "big" operators (Section 3.1, Graph Optimization), says that
 * backward is the symbolic derivative of forward (Section 2.1) and that the
 * CNN benchmark's run time is spent in these kernels (Section 4, Raw
 * performance).  It prints no formula, so the direct sum below is the
 * definition; backward-data and backward-weight are the exact adjoints of the
 * forward map in x and in w (the map is bilinear).
 *
 * Conventions (readings of what the paper leaves open):
 *   - cross-correlation, no filter flip;
 *   - P = floor((H + 2*pad - R)/stride) + 1, Q likewise with W and S;
 *   - x outside [0,H)x[0,W) reads as 0;
 *   - one stride and one pad for both axes, dilation 1, groups 1, no bias;
 *   - tensors are dense row-major: x[N][C][H][W], w[K][C][R][S], y[N][K][P][Q].
 *
 * Inputs are float because the values handed to the GPU path are fp32 or bf16,
 * both of which a float holds exactly; every product and sum is in double.
 *
 * Every full-tensor routine is a literal seven-deep loop nest.  OpenMP is put
 * on the outermost loop(s) only, chosen so that threads write disjoint outputs.
 * The *_at routines evaluate single output elements (gather form) and also
 * return D = sum |a|*|b| over the same taps, the denominator of the error
 * metric.  The full-tensor backward routines are scatter form, so the two
 * families do not share index arithmetic and are tested against each other.
 */
#include <math.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef long long i64;

static int out_dim(int in, int filt, int stride, int pad)
{
    return (in + 2 * pad - filt) / stride + 1;
}

int orc_out_dim(int in, int filt, int stride, int pad)
{
    return out_dim(in, filt, stride, pad);
}

/* y[n,k,p,q] = sum_{c,r,s} x[n,c,p*stride-pad+r,q*stride-pad+s] * w[k,c,r,s] */
void orc_conv2d_fwd(int N, int C, int H, int W, int K, int R, int S,
                    int stride, int pad,
                    const float *x, const float *w, double *y)
{
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                const int h = p * stride - pad + r;
                                const int v = q * stride - pad + s;
                                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                                acc += (double)x[(((i64)n * C + c) * H + h) * W + v] *
                                       (double)w[(((i64)k * C + c) * R + r) * S + s];
                            }
                    y[(((i64)n * K + k) * P + p) * Q + q] = acc;
                }
}

/* dx[n,c,h,v] += dy[n,k,p,q] * w[k,c,r,s] for every tap that lands on (h,v);
 * positions no tap reaches stay exactly 0. */
void orc_conv2d_bwd_data(int N, int C, int H, int W, int K, int R, int S,
                         int stride, int pad,
                         const float *dy, const float *w, double *dx)
{
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
    memset(dx, 0, sizeof(double) * (size_t)N * C * H * W);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int k = 0; k < K; ++k)
                for (int p = 0; p < P; ++p)
                    for (int q = 0; q < Q; ++q)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                const int h = p * stride - pad + r;
                                const int v = q * stride - pad + s;
                                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                                dx[(((i64)n * C + c) * H + h) * W + v] +=
                                    (double)dy[(((i64)n * K + k) * P + p) * Q + q] *
                                    (double)w[(((i64)k * C + c) * R + r) * S + s];
                            }
}

/* dw[k,c,r,s] += dy[n,k,p,q] * x[n,c,p*stride-pad+r,q*stride-pad+s] */
void orc_conv2d_bwd_weight(int N, int C, int H, int W, int K, int R, int S,
                           int stride, int pad,
                           const float *x, const float *dy, double *dw)
{
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
    memset(dw, 0, sizeof(double) * (size_t)K * C * R * S);
#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < C; ++c)
            for (int n = 0; n < N; ++n)
                for (int p = 0; p < P; ++p)
                    for (int q = 0; q < Q; ++q)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                const int h = p * stride - pad + r;
                                const int v = q * stride - pad + s;
                                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                                dw[(((i64)k * C + c) * R + r) * S + s] +=
                                    (double)dy[(((i64)n * K + k) * P + p) * Q + q] *
                                    (double)x[(((i64)n * C + c) * H + h) * W + v];
                            }
}

/* ---- single-element evaluators (gather form) ---------------------------- */
/* idx[i] is the flat row-major index into the output tensor; val[i] receives
 * the exact sum, den[i] the sum of |a|*|b| over the same taps. */

void orc_conv2d_fwd_at(int N, int C, int H, int W, int K, int R, int S,
                       int stride, int pad,
                       const float *x, const float *w,
                       i64 count, const i64 *idx, double *val, double *den)
{
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
    (void)N;
#pragma omp parallel for schedule(dynamic, 64)
    for (i64 i = 0; i < count; ++i) {
        i64 t = idx[i];
        const int q = (int)(t % Q); t /= Q;
        const int p = (int)(t % P); t /= P;
        const int k = (int)(t % K); t /= K;
        const int n = (int)t;
        double acc = 0.0, mag = 0.0;
        for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s) {
                    const int h = p * stride - pad + r;
                    const int v = q * stride - pad + s;
                    if (h < 0 || h >= H || v < 0 || v >= W) continue;
                    const double a = x[(((i64)n * C + c) * H + h) * W + v];
                    const double b = w[(((i64)k * C + c) * R + r) * S + s];
                    acc += a * b;
                    mag += fabs(a) * fabs(b);
                }
        val[i] = acc;
        den[i] = mag;
    }
}

/* dx[n,c,h,v] = sum over (k,r,s) with (h+pad-r) and (v+pad-s) divisible by
 * stride and the quotients p,q inside the output, of dy[n,k,p,q]*w[k,c,r,s]. */
void orc_conv2d_bwd_data_at(int N, int C, int H, int W, int K, int R, int S,
                            int stride, int pad,
                            const float *dy, const float *w,
                            i64 count, const i64 *idx, double *val, double *den)
{
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
    (void)N;
#pragma omp parallel for schedule(dynamic, 64)
    for (i64 i = 0; i < count; ++i) {
        i64 t = idx[i];
        const int v = (int)(t % W); t /= W;
        const int h = (int)(t % H); t /= H;
        const int c = (int)(t % C); t /= C;
        const int n = (int)t;
        double acc = 0.0, mag = 0.0;
        for (int k = 0; k < K; ++k)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s) {
                    const int hp = h + pad - r, vq = v + pad - s;
                    if (hp < 0 || vq < 0) continue;
                    if (hp % stride != 0 || vq % stride != 0) continue;
                    const int p = hp / stride, q = vq / stride;
                    if (p >= P || q >= Q) continue;
                    const double a = dy[(((i64)n * K + k) * P + p) * Q + q];
                    const double b = w[(((i64)k * C + c) * R + r) * S + s];
                    acc += a * b;
                    mag += fabs(a) * fabs(b);
                }
        val[i] = acc;
        den[i] = mag;
    }
}

void orc_conv2d_bwd_weight_at(int N, int C, int H, int W, int K, int R, int S,
                              int stride, int pad,
                              const float *x, const float *dy,
                              i64 count, const i64 *idx, double *val, double *den)
{
    const int P = out_dim(H, R, stride, pad), Q = out_dim(W, S, stride, pad);
#pragma omp parallel for schedule(dynamic, 4)
    for (i64 i = 0; i < count; ++i) {
        i64 t = idx[i];
        const int s = (int)(t % S); t /= S;
        const int r = (int)(t % R); t /= R;
        const int c = (int)(t % C); t /= C;
        const int k = (int)t;
        double acc = 0.0, mag = 0.0;
        for (int n = 0; n < N; ++n)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const int h = p * stride - pad + r;
                    const int v = q * stride - pad + s;
                    if (h < 0 || h >= H || v < 0 || v >= W) continue;
                    const double a = dy[(((i64)n * K + k) * P + p) * Q + q];
                    const double b = x[(((i64)n * C + c) * H + h) * W + v];
                    acc += a * b;
                    mag += fabs(a) * fabs(b);
                }
        val[i] = acc;
        den[i] = mag;
    }
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
