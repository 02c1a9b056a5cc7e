// Softmax output layer: p[n][k] = exp(z[n][k] - max_j z[n][j]) / sum_j exp(...), and the gradient of the
// cross-entropy against integer labels, (p - onehot(label)) * scale.  One workgroup per row; fp32
// arithmetic whatever the storage type; row maximum and sum reduced through LDS in a fixed order.
#include "mxc_internal.h"

namespace mxc {
namespace {

constexpr int SM_THREADS = 256;

__device__ __forceinline__ float block_reduce(float v, float *red, bool is_max)
{
    red[threadIdx.x] = v;
    __syncthreads();
    for (int half = SM_THREADS / 2; half > 0; half >>= 1) {
        if ((int)threadIdx.x < half) red[threadIdx.x] = is_max ? fmaxf(red[threadIdx.x], red[threadIdx.x + half])
                                                               : red[threadIdx.x] + red[threadIdx.x + half];
        __syncthreads();
    }
    const float r = red[0];
    __syncthreads();
    return r;
}

template <typename T>
__global__ __launch_bounds__(SM_THREADS) void softmax_fwd_kernel(const T *__restrict__ z, T *__restrict__ p, int K)
{
    __shared__ float red[SM_THREADS];
    const T *zr = z + (size_t)blockIdx.x * K;
    T *pr = p + (size_t)blockIdx.x * K;
    float mx = -3.0e38f;
    for (int k = threadIdx.x; k < K; k += SM_THREADS) mx = fmaxf(mx, load_f32(zr + k));
    mx = block_reduce(mx, red, true);
    float sum = 0.f;
    for (int k = threadIdx.x; k < K; k += SM_THREADS) sum += expf(load_f32(zr + k) - mx);
    sum = block_reduce(sum, red, false);
    const float inv = 1.f / sum;
    for (int k = threadIdx.x; k < K; k += SM_THREADS) store_f32(pr + k, expf(load_f32(zr + k) - mx) * inv);
}

template <typename T>
__global__ __launch_bounds__(SM_THREADS) void softmax_xent_bwd_kernel(const T *__restrict__ p, const int *__restrict__ labels,
                                                                      T *__restrict__ dz, int K, float scale)
{
    const T *pr = p + (size_t)blockIdx.x * K;
    T *dr = dz + (size_t)blockIdx.x * K;
    const int label = labels[blockIdx.x];
    for (int k = threadIdx.x; k < K; k += SM_THREADS) store_f32(dr + k, (load_f32(pr + k) - (k == label ? 1.f : 0.f)) * scale);
}

}  // namespace

int softmax_fwd(int N, int K, int dtype, const void *z, void *p, hipStream_t st)
{
    if (dtype == MXC_BF16) hipLaunchKernelGGL(softmax_fwd_kernel<bf16_t>, dim3((unsigned)N), dim3(SM_THREADS), 0, st, (const bf16_t *)z, (bf16_t *)p, K);
    else hipLaunchKernelGGL(softmax_fwd_kernel<float>, dim3((unsigned)N), dim3(SM_THREADS), 0, st, (const float *)z, (float *)p, K);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

int softmax_xent_bwd(int N, int K, int dtype, const void *p, const int *labels, void *dz, float scale, hipStream_t st)
{
    if (dtype == MXC_BF16)
        hipLaunchKernelGGL(softmax_xent_bwd_kernel<bf16_t>, dim3((unsigned)N), dim3(SM_THREADS), 0, st, (const bf16_t *)p, labels,
                           (bf16_t *)dz, K, scale);
    else
        hipLaunchKernelGGL(softmax_xent_bwd_kernel<float>, dim3((unsigned)N), dim3(SM_THREADS), 0, st, (const float *)p, labels,
                           (float *)dz, K, scale);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

}  // namespace mxc
