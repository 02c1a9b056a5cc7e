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

// NHWC, K a multiple of VEC (16 bytes of elements) and at most 256*VEC: thread t owns the 16-byte
// channel chunk t % (K/VEC) of the rows  r0 + t / (K/VEC) + i * groups;  four rows are in flight per
// thread.  The row groups are then added in LDS in ascending order.
template <typename T, int VEC>
__global__ __launch_bounds__(BG_THREADS) void bias_grad_rows_vec_kernel(const T *__restrict__ dy, float *__restrict__ partial,
                                                                        long long rows, int K, int rows_per_wg)
{
    __shared__ float red[BG_THREADS * VEC];
    const int chunks = K / VEC, groups = BG_THREADS / chunks;
    const int chunk = threadIdx.x % chunks, grp = threadIdx.x / chunks;
    const long long r0 = (long long)blockIdx.x * rows_per_wg;
    long long r1 = r0 + rows_per_wg;
    if (r1 > rows) r1 = rows;
    float acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = 0.f;
    auto add = [&](const uint4 &v) {
        if constexpr (sizeof(T) == 2) {
            const uint32_t u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[2 * e] += __uint_as_float(u[e] << 16);
                acc[2 * e + 1] += __uint_as_float(u[e] & 0xFFFF0000u);
            }
        } else {
            acc[0] += __uint_as_float(v.x); acc[1] += __uint_as_float(v.y);
            acc[2] += __uint_as_float(v.z); acc[3] += __uint_as_float(v.w);
        }
    };
    if (grp < groups) {
        const uint4 *base = reinterpret_cast<const uint4 *>(dy) + chunk;      // row r: base[r * chunks]
        long long r = r0 + grp;
        for (; r + 3LL * groups < r1; r += 4LL * groups) {
            const uint4 a = base[r * chunks], b = base[(r + groups) * chunks], c = base[(r + 2LL * groups) * chunks],
                        d = base[(r + 3LL * groups) * chunks];
            add(a); add(b); add(c); add(d);
        }
        for (; r < r1; r += groups) add(base[r * chunks]);
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) red[threadIdx.x * VEC + e] = acc[e];
    __syncthreads();
    if (grp == 0) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            float s = 0.f;
            for (int g = 0; g < groups; ++g) s += red[(g * chunks + chunk) * VEC + e];
            partial[(size_t)blockIdx.x * K + chunk * VEC + e] = s;
        }
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

// db[k] = sum of the partial vectors, in a fixed order: a workgroup of 1024 threads owns 32 columns;
// its 32 thread groups each add every 32nd partial vector, then the 32 sums are added in ascending
// order.
constexpr int BG_SUM_THREADS = 1024;
__global__ __launch_bounds__(BG_SUM_THREADS) void bias_grad_sum_kernel(const float *__restrict__ partial, float *__restrict__ db, int K,
                                                                       int parts)
{
    __shared__ float red[BG_SUM_THREADS];
    constexpr int GROUPS = BG_SUM_THREADS / 32;
    const int col = threadIdx.x % 32, grp = threadIdx.x / 32;
    const int k = blockIdx.x * 32 + col;
    float acc = 0.f;
    if (k < K)
        for (int i = grp; i < parts; i += GROUPS) acc += partial[(size_t)i * K + k];
    red[threadIdx.x] = acc;
    __syncthreads();
    if (grp == 0 && k < K) {
        float s = 0.f;
        for (int g = 0; g < GROUPS; ++g) s += red[g * 32 + col];
        db[k] = s;
    }
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
    if (parts > 1024) parts = 1024;
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
        const int vec = dtype == MXC_BF16 ? 8 : 4;
        const bool vector = K % vec == 0 && K / vec <= BG_THREADS;
        if (dtype == MXC_BF16) {
            if (vector)
                hipLaunchKernelGGL((bias_grad_rows_vec_kernel<bf16_t, 8>), dim3((unsigned)parts), dim3(BG_THREADS), 0, st,
                                   (const bf16_t *)dy, partial, rows, K, rows_per_wg);
            else
                hipLaunchKernelGGL(bias_grad_rows_kernel<bf16_t>, dim3((unsigned)parts), dim3(BG_THREADS), 0, st, (const bf16_t *)dy,
                                   partial, rows, K, rows_per_wg);
        } else {
            if (vector)
                hipLaunchKernelGGL((bias_grad_rows_vec_kernel<float, 4>), dim3((unsigned)parts), dim3(BG_THREADS), 0, st,
                                   (const float *)dy, partial, rows, K, rows_per_wg);
            else
                hipLaunchKernelGGL(bias_grad_rows_kernel<float>, dim3((unsigned)parts), dim3(BG_THREADS), 0, st, (const float *)dy,
                                   partial, rows, K, rows_per_wg);
        }
    }
    if (hipGetLastError() != hipSuccess) return MXC_ERR_LAUNCH;
    hipLaunchKernelGGL(bias_grad_sum_kernel, dim3((unsigned)((K + 31) / 32)), dim3(BG_SUM_THREADS), 0, st, partial, db, K, parts);
    return ok();
}

}  // namespace mxc
