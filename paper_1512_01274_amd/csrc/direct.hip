// Direct (one thread per output element) convolution kernels.
//
// These cover every shape and both element types and are the path for fp32 and
// for shapes the MFMA kernels do not take.  Working layout: activations NHWC,
// filters KRSC, fp32 accumulation in a fixed order (deterministic).
#include "mxc_internal.h"

namespace mxc {

namespace {

// y[n,p,q,k] = sum_{r,s,c} x[n,p*st-pad+r,q*st-pad+s,c] * w[k,r,s,c]
template <typename T>
__global__ __launch_bounds__(256) void direct_fwd_kernel(ConvShape s, const T *__restrict__ x, const T *__restrict__ w,
                                                         T *__restrict__ y, size_t total, const float *__restrict__ bias, int relu)
{
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    size_t t = gid;
    const int k = (int)(t % s.K); t /= s.K;
    const int q = (int)(t % s.Q); t /= s.Q;
    const int p = (int)(t % s.P); t /= s.P;
    const int n = (int)t;
    float acc = 0.f;
    for (int r = 0; r < s.R; ++r) {
        const int h = p * s.stride - s.pad + r;
        if (h < 0 || h >= s.H) continue;
        for (int ss = 0; ss < s.S; ++ss) {
            const int v = q * s.stride - s.pad + ss;
            if (v < 0 || v >= s.W) continue;
            const T *xp = x + (((size_t)n * s.H + h) * s.W + v) * s.C;
            const T *wp = w + (((size_t)k * s.R + r) * s.S + ss) * s.C;
            for (int c = 0; c < s.C; ++c) acc = fmaf(load_f32(xp + c), load_f32(wp + c), acc);
        }
    }
    if (bias != nullptr) acc += bias[k];
    if (relu) acc = fmaxf(acc, 0.f);
    store_f32(y + gid, acc);
}

// dx[n,h,v,c] = sum over taps (r,s) with (h+pad-r)%st==0, (v+pad-s)%st==0, p,q in range, and k.
template <typename T>
__global__ __launch_bounds__(256) void direct_bwd_data_kernel(ConvShape s, const T *__restrict__ dy,
                                                              const T *__restrict__ w, T *__restrict__ dx, size_t total,
                                                              const T *__restrict__ mask)
{
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    size_t t = gid;
    const int c = (int)(t % s.C); t /= s.C;
    const int v = (int)(t % s.W); t /= s.W;
    const int h = (int)(t % s.H); t /= s.H;
    const int n = (int)t;
    float acc = 0.f;
    for (int r = 0; r < s.R; ++r) {
        const int hp = h + s.pad - r;
        if (hp < 0 || hp % s.stride != 0) continue;
        const int p = hp / s.stride;
        if (p >= s.P) continue;
        for (int ss = 0; ss < s.S; ++ss) {
            const int vq = v + s.pad - ss;
            if (vq < 0 || vq % s.stride != 0) continue;
            const int q = vq / s.stride;
            if (q >= s.Q) continue;
            const T *dyp = dy + (((size_t)n * s.P + p) * s.Q + q) * s.K;
            const T *wp = w + ((size_t)r * s.S + ss) * s.C + c;
            const size_t wk = (size_t)s.R * s.S * s.C;
            for (int k = 0; k < s.K; ++k) acc = fmaf(load_f32(dyp + k), load_f32(wp + (size_t)k * wk), acc);
        }
    }
    if (mask != nullptr && !mask_keeps(mask + gid)) acc = 0.f;
    store_f32(dx + gid, acc);
}

// partial[split][k,r,s,c] = sum over the split's pixel range of dy[n,p,q,k] * x[n,h,v,c]
template <typename T>
__global__ __launch_bounds__(256) void direct_bwd_weight_kernel(ConvShape s, const T *__restrict__ x,
                                                                const T *__restrict__ dy, float *__restrict__ partial,
                                                                int pix_per_split)
{
    const int wtotal = s.K * s.R * s.S * s.C;
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= wtotal) return;
    int t = gid;
    const int c = t % s.C; t /= s.C;
    const int ss = t % s.S; t /= s.S;
    const int r = t % s.R; t /= s.R;
    const int k = t;
    const long long npq = (long long)s.N * s.P * s.Q;
    const long long m0 = (long long)blockIdx.y * pix_per_split;
    long long m1 = m0 + pix_per_split;
    if (m1 > npq) m1 = npq;
    float acc = 0.f;
    for (long long m = m0; m < m1; ++m) {
        const int q = (int)(m % s.Q);
        const int p = (int)((m / s.Q) % s.P);
        const int n = (int)(m / ((long long)s.P * s.Q));
        const int h = p * s.stride - s.pad + r, v = q * s.stride - s.pad + ss;
        if (h < 0 || h >= s.H || v < 0 || v >= s.W) continue;
        acc = fmaf(load_f32(dy + (size_t)m * s.K + k), load_f32(x + (((size_t)n * s.H + h) * s.W + v) * s.C + c), acc);
    }
    partial[(size_t)blockIdx.y * wtotal + gid] = acc;
}

// dw[i] = partial[0][i] + partial[1][i] + ... in that order (OUT = bf16_t: the fp32 sum rounded once)
template <typename OUT>
__global__ __launch_bounds__(256) void sum_splits_kernel(const float *__restrict__ partial, OUT *__restrict__ dw,
                                                         int wtotal, int splits)
{
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= wtotal) return;
    float acc = 0.f;
    for (int i = 0; i < splits; ++i) acc += partial[(size_t)i * wtotal + gid];
    store_f32(dw + gid, acc);
}

inline int ok() { return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH; }

}  // namespace

int direct_fwd(const ConvShape &s, int dtype, const void *x, const void *w, void *y, hipStream_t st, const PostOp &post)
{
    const size_t total = (size_t)s.N * s.P * s.Q * s.K;
    const size_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return MXC_ERR_SHAPE;
    if (dtype == MXC_BF16)
        hipLaunchKernelGGL(direct_fwd_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, st, s, (const bf16_t *)x,
                           (const bf16_t *)w, (bf16_t *)y, total, post.bias, post.relu);
    else
        hipLaunchKernelGGL(direct_fwd_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, st, s, (const float *)x,
                           (const float *)w, (float *)y, total, post.bias, post.relu);
    return ok();
}

int direct_bwd_data(const ConvShape &s, int dtype, const void *dy, const void *w, void *dx, hipStream_t st, const PostOp &post)
{
    const size_t total = (size_t)s.N * s.H * s.W * s.C;
    const size_t blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFull) return MXC_ERR_SHAPE;
    if (dtype == MXC_BF16)
        hipLaunchKernelGGL(direct_bwd_data_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, st, s,
                           (const bf16_t *)dy, (const bf16_t *)w, (bf16_t *)dx, total, (const bf16_t *)post.mask);
    else
        hipLaunchKernelGGL(direct_bwd_data_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, st, s,
                           (const float *)dy, (const float *)w, (float *)dx, total, (const float *)post.mask);
    return ok();
}

int direct_bwd_weight_splits(const ConvShape &s)
{
    // Enough splits to occupy the chip when the filter is small, never more than the pixel count.
    const long long wtotal = (long long)s.K * s.R * s.S * s.C;
    const long long npq = (long long)s.N * s.P * s.Q;
    long long blocks = (wtotal + 255) / 256;
    long long splits = (2048 + blocks - 1) / blocks;
    if (splits > 256) splits = 256;
    if (splits > npq) splits = npq;
    if (splits < 1) splits = 1;
    return (int)splits;
}

int direct_bwd_weight(const ConvShape &s, int dtype, const void *x, const void *dy, void *dw, bool dw_bf16, float *partial,
                      int splits, hipStream_t st)
{
    const long long wtotal_ll = (long long)s.K * s.R * s.S * s.C;
    if (wtotal_ll > 0x7FFFFFFFll) return MXC_ERR_SHAPE;
    const int wtotal = (int)wtotal_ll;
    const long long npq = (long long)s.N * s.P * s.Q;
    const long long pps = (npq + splits - 1) / splits;
    if (pps > 0x7FFFFFFFll) return MXC_ERR_SHAPE;
    dim3 grid((unsigned)((wtotal + 255) / 256), (unsigned)splits), block(256);
    if (dtype == MXC_BF16)
        hipLaunchKernelGGL(direct_bwd_weight_kernel<bf16_t>, grid, block, 0, st, s, (const bf16_t *)x,
                           (const bf16_t *)dy, partial, (int)pps);
    else
        hipLaunchKernelGGL(direct_bwd_weight_kernel<float>, grid, block, 0, st, s, (const float *)x, (const float *)dy,
                           partial, (int)pps);
    if (ok() != MXC_OK) return MXC_ERR_LAUNCH;
    if (dw_bf16)
        hipLaunchKernelGGL(sum_splits_kernel<bf16_t>, dim3((unsigned)((wtotal + 255) / 256)), block, 0, st, partial, (bf16_t *)dw,
                           wtotal, splits);
    else
        hipLaunchKernelGGL(sum_splits_kernel<float>, dim3((unsigned)((wtotal + 255) / 256)), block, 0, st, partial, (float *)dw,
                           wtotal, splits);
    return ok();
}

}  // namespace mxc
