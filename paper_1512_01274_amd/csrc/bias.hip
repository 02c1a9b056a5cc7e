// Bias gradient: db[k] = sum over images and pixels of dy[n, k, p, q], fp32, deterministic.
//
// HBM-bound (dy is read once).  Two steps, both in a fixed order: every workgroup sums a block of
// rows of the [rows][K] view (NHWC) or one (n, k) plane (NCHW) into a partial vector, then one
// kernel adds the partial vectors in ascending order.
#include "mxc_internal.h"

namespace mxc {
namespace {

constexpr int BG_THREADS = 256;

// NHWC: dy is [rows = N*P*Q][K].  Thread t of a workgroup owns columns t, t+256, ... for the
// workgroup's rows_per_wg consecutive rows; lanes read consecutive channels (coalesced).
template <typename T>
__global__ __launch_bounds__(BG_THREADS) void bias_grad_rows_kernel(const T *__restrict__ dy, float *__restrict__ partial,
                                                                    long long rows, int K, int rows_per_wg)
{
    const long long r0 = (long long)blockIdx.x * rows_per_wg;
    long long r1 = r0 + rows_per_wg;
    if (r1 > rows) r1 = rows;
    for (int k = threadIdx.x; k < K; k += BG_THREADS) {
        float acc = 0.f;
        for (long long r = r0; r < r1; ++r) acc += load_f32(dy + r * K + k);
        partial[(size_t)blockIdx.x * K + k] = acc;
    }
}

// NHWC with few channels (K <= 128, a power of two): a workgroup's threads form 256/K row groups so
// that all lanes stay busy; the row groups are then added in LDS in a fixed order.
template <typename T>
__global__ __launch_bounds__(BG_THREADS) void bias_grad_rows_narrow_kernel(const T *__restrict__ dy, float *__restrict__ partial,
                                                                           long long rows, int K, int rows_per_wg)
{
    __shared__ float red[BG_THREADS];
    const int groups = BG_THREADS / K;
    const int k = threadIdx.x % K, grp = threadIdx.x / K;
    const long long r0 = (long long)blockIdx.x * rows_per_wg;
    long long r1 = r0 + rows_per_wg;
    if (r1 > rows) r1 = rows;
    float acc = 0.f;
    for (long long r = r0 + grp; r < r1; r += groups) acc += load_f32(dy + r * K + k);
    red[threadIdx.x] = acc;
    __syncthreads();
    if (grp == 0) {
        float s = 0.f;
        for (int g = 0; g < groups; ++g) s += red[g * K + k];
        partial[(size_t)blockIdx.x * K + k] = s;
    }
}

// NCHW: dy is [N][K][PQ]; workgroup (n*K + k) sums its plane; partial is [N][K]
template <typename T>
__global__ __launch_bounds__(BG_THREADS) void bias_grad_planes_kernel(const T *__restrict__ dy, float *__restrict__ partial, int PQ)
{
    __shared__ float red[BG_THREADS];
    const T *src = dy + (size_t)blockIdx.x * PQ;
    float acc = 0.f;
    for (int i = threadIdx.x; i < PQ; i += BG_THREADS) acc += load_f32(src + i);
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int half = BG_THREADS / 2; half > 0; half >>= 1) {
        if ((int)threadIdx.x < half) red[threadIdx.x] += red[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
}

__global__ __launch_bounds__(BG_THREADS) void bias_grad_sum_kernel(const float *__restrict__ partial, float *__restrict__ db, int K,
                                                                   int parts)
{
    const int k = blockIdx.x * BG_THREADS + threadIdx.x;
    if (k >= K) return;
    float acc = 0.f;
    for (int i = 0; i < parts; ++i) acc += partial[(size_t)i * K + k];
    db[k] = acc;
}

inline int ok() { return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH; }

}  // namespace

// number of partial vectors (each K floats) the first step produces
int bias_grad_parts(long long N, int K, long long PQ, int layout)
{
    if (layout == MXC_NCHW) return (int)N;
    (void)K;
    const long long rows = N * PQ;
    long long parts = (rows + 255) / 256;      // at least 256 rows per workgroup
    if (parts > 2048) parts = 2048;
    return (int)(parts < 1 ? 1 : parts);
}

int bias_grad(long long N, int K, long long PQ, int dtype, int layout, const void *dy, float *db, float *partial, hipStream_t st)
{
    const int parts = bias_grad_parts(N, K, PQ, layout);
    if (layout == MXC_NCHW) {
        if (N * K > 0x7FFFFFFFll || PQ > 0x7FFFFFFFll) return MXC_ERR_SHAPE;
        if (dtype == MXC_BF16)
            hipLaunchKernelGGL(bias_grad_planes_kernel<bf16_t>, dim3((unsigned)(N * K)), dim3(BG_THREADS), 0, st, (const bf16_t *)dy,
                               partial, (int)PQ);
        else
            hipLaunchKernelGGL(bias_grad_planes_kernel<float>, dim3((unsigned)(N * K)), dim3(BG_THREADS), 0, st, (const float *)dy,
                               partial, (int)PQ);
    } else {
        const long long rows = N * PQ;
        const int rows_per_wg = (int)((rows + parts - 1) / parts);
        const bool narrow = K <= 128 && (K & (K - 1)) == 0;
        if (dtype == MXC_BF16) {
            if (narrow)
                hipLaunchKernelGGL(bias_grad_rows_narrow_kernel<bf16_t>, dim3((unsigned)parts), dim3(BG_THREADS), 0, st,
                                   (const bf16_t *)dy, partial, rows, K, rows_per_wg);
            else
                hipLaunchKernelGGL(bias_grad_rows_kernel<bf16_t>, dim3((unsigned)parts), dim3(BG_THREADS), 0, st, (const bf16_t *)dy,
                                   partial, rows, K, rows_per_wg);
        } else {
            if (narrow)
                hipLaunchKernelGGL(bias_grad_rows_narrow_kernel<float>, dim3((unsigned)parts), dim3(BG_THREADS), 0, st,
                                   (const float *)dy, partial, rows, K, rows_per_wg);
            else
                hipLaunchKernelGGL(bias_grad_rows_kernel<float>, dim3((unsigned)parts), dim3(BG_THREADS), 0, st, (const float *)dy,
                                   partial, rows, K, rows_per_wg);
        }
    }
    if (hipGetLastError() != hipSuccess) return MXC_ERR_LAUNCH;
    hipLaunchKernelGGL(bias_grad_sum_kernel, dim3((unsigned)((K + BG_THREADS - 1) / BG_THREADS)), dim3(BG_THREADS), 0, st, partial, db,
                       K, parts);
    return ok();
}

}  // namespace mxc
