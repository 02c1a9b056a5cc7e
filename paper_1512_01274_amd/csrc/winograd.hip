// 3x3 stride-1 forward convolution in the transform domain, F(2x2, 3x3): another algorithm for the layer's
// "forward" evaluation (paper Section 2.1), beside the implicit GEMM.
//
// With the usual matrices
//     G  = [1 0 0; .5 .5 .5; .5 -.5 .5; 0 0 1]       (4x3, filter)
//     Bt = [1 0 -1 0; 0 1 1 0; 0 -1 1 0; 0 1 0 -1]   (4x4, input)
//     At = [1 1 1 0; 0 1 -1 -1]                      (2x4, output)
// a 2x2 block of outputs is  Y = At [ sum_c (G g_c Gt) .* (Bt d_c B) ] A,  d_c the 4x4 input patch of channel c
// that the block reads: 16 multiplications per channel and block instead of 36.  The sum over channels is, for
// each of the 16 positions xi of the 4x4 product, a plain GEMM  M_xi[tile][k] = sum_c V_xi[tile][c] * U_xi[k][c]:
//   1. filter transform   U[xi][k][c]    = (G g Gt)[xi]          bf16 (rounded once)
//   2. input transform    V[xi][tile][c] = (Bt d B)[xi]          bf16 (rounded once), zero padding applied on load
//   3. 16 GEMMs on the matrix cores, fp32 sums kept unrounded (igemm_gemm_f32)
//   4. output transform   y = At M A (+ bias, ReLU), rounded once to bf16
// Steps 1, 2 and 4 are elementwise-sized kernels: one thread per (tile or filter, 4 channels), 8-byte accesses.
// The error of this form is that of the two bf16 roundings in the transform domain: at most
// 2^-8 * sum over the M entries a result combines of sum_c |U||V| (the tests evaluate that bound on the host).
#include <stdio.h>

#include "mxc_internal.h"

namespace mxc {

namespace {

__device__ __forceinline__ void unpack4(uint2 v, float f[4])
{
    f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
    f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
}

// U[xi][k][c] for xi = i*4 + j; one thread per (k, c)
__global__ __launch_bounds__(256) void wino_filter_kernel(const bf16_t *__restrict__ w, bf16_t *__restrict__ U, int K, int C)
{
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= K * C) return;
    const int c = gid % C, k = gid / C;
    float g[3][3];
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s = 0; s < 3; ++s) g[r][s] = bf16_to_f32(w[((size_t)(k * 3 + r) * 3 + s) * C + c]);
    float t[4][3];
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        t[0][s] = g[0][s];
        t[1][s] = 0.5f * (g[0][s] + g[1][s] + g[2][s]);
        t[2][s] = 0.5f * (g[0][s] - g[1][s] + g[2][s]);
        t[3][s] = g[2][s];
    }
    const size_t plane = (size_t)K * C;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float u0 = t[i][0], u1 = 0.5f * (t[i][0] + t[i][1] + t[i][2]), u2 = 0.5f * (t[i][0] - t[i][1] + t[i][2]), u3 = t[i][2];
        U[(size_t)(i * 4 + 0) * plane + gid] = f32_to_bf16(u0);
        U[(size_t)(i * 4 + 1) * plane + gid] = f32_to_bf16(u1);
        U[(size_t)(i * 4 + 2) * plane + gid] = f32_to_bf16(u2);
        U[(size_t)(i * 4 + 3) * plane + gid] = f32_to_bf16(u3);
    }
}

// V[xi][tile][c]; tile = (n, tp, tq) reads input rows 2tp-pad .. +3, columns 2tq-pad .. +3; one thread per (tile, 4 channels)
__global__ __launch_bounds__(256) void wino_input_kernel(const bf16_t *__restrict__ x, bf16_t *__restrict__ V, long long tiles, int TP,
                                                         int TQ, int H, int W, int C, int pad)
{
    const int c4n = C / 4;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= tiles * c4n) return;
    const int c = (int)(gid % c4n) * 4;
    const long long tile = gid / c4n;
    const int tq = (int)(tile % TQ), tp = (int)((tile / TQ) % TP);
    const long long n = tile / ((long long)TQ * TP);
    const int h0 = 2 * tp - pad, w0 = 2 * tq - pad;
    // column transform while loading: t[i][j] = (Bt d)[i][j]
    float t[4][4][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float d[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int h = h0 + i, wc = w0 + j;
            uint2 v = make_uint2(0u, 0u);
            if (h >= 0 && h < H && wc >= 0 && wc < W) v = *reinterpret_cast<const uint2 *>(x + (((size_t)n * H + h) * W + wc) * C + c);
            unpack4(v, d[i]);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            t[0][j][e] = d[0][e] - d[2][e];
            t[1][j][e] = d[1][e] + d[2][e];
            t[2][j][e] = d[2][e] - d[1][e];
            t[3][j][e] = d[1][e] - d[3][e];
        }
    }
    const size_t plane = (size_t)tiles * C;
    bf16_t *dst = V + (size_t)tile * C + c;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float o[4][4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            o[0][e] = t[i][0][e] - t[i][2][e];
            o[1][e] = t[i][1][e] + t[i][2][e];
            o[2][e] = t[i][2][e] - t[i][1][e];
            o[3][e] = t[i][1][e] - t[i][3][e];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            *reinterpret_cast<uint2 *>(dst + (size_t)(i * 4 + j) * plane) = make_uint2(pack_bf16x2(o[j][0], o[j][1]), pack_bf16x2(o[j][2], o[j][3]));
    }
}

// y = At M A (+ bias, ReLU); one thread per (tile, 4 output channels)
__global__ __launch_bounds__(256) void wino_output_kernel(const float *__restrict__ M, bf16_t *__restrict__ y, long long tiles, int TP,
                                                          int TQ, int P, int Q, int K, const float *__restrict__ bias, int relu)
{
    const int k4n = K / 4;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= tiles * k4n) return;
    const int k = (int)(gid % k4n) * 4;
    const long long tile = gid / k4n;
    const int tq = (int)(tile % TQ), tp = (int)((tile / TQ) % TP);
    const long long n = tile / ((long long)TQ * TP);
    const size_t plane = (size_t)tiles * K;
    const float *src = M + (size_t)tile * K + k;
    float r[2][4][4];       // row transform while loading: r[a][j] = (At m)[a][j]
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float4 m[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) m[i] = *reinterpret_cast<const float4 *>(src + (size_t)(i * 4 + j) * plane);
        r[0][j][0] = m[0].x + m[1].x + m[2].x; r[1][j][0] = m[1].x - m[2].x - m[3].x;
        r[0][j][1] = m[0].y + m[1].y + m[2].y; r[1][j][1] = m[1].y - m[2].y - m[3].y;
        r[0][j][2] = m[0].z + m[1].z + m[2].z; r[1][j][2] = m[1].z - m[2].z - m[3].z;
        r[0][j][3] = m[0].w + m[1].w + m[2].w; r[1][j][3] = m[1].w - m[2].w - m[3].w;
    }
    float b4[4] = {0.f, 0.f, 0.f, 0.f};
    if (bias != nullptr) { b4[0] = bias[k]; b4[1] = bias[k + 1]; b4[2] = bias[k + 2]; b4[3] = bias[k + 3]; }
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const int p = 2 * tp + a;
        if (p >= P) continue;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int q = 2 * tq + b;
            if (q >= Q) continue;
            float o[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                o[e] = (b == 0 ? r[a][0][e] + r[a][1][e] + r[a][2][e] : r[a][1][e] - r[a][2][e] - r[a][3][e]) + b4[e];
                if (relu) o[e] = fmaxf(o[e], 0.f);
            }
            *reinterpret_cast<uint2 *>(y + (((size_t)n * P + p) * Q + q) * K + k) = make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
        }
    }
}

inline long long tile_count(const ConvShape &s) { return (long long)s.N * ((s.P + 1) / 2) * ((s.Q + 1) / 2); }
inline int ok() { return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH; }

}  // namespace

bool winograd_supported(const ConvShape &s)
{
    const long long T = tile_count(s);
    return s.R == 3 && s.S == 3 && s.stride == 1 && s.C % 8 == 0 && s.K % 8 == 0 && igemm_gemm_f32_supported(T, s.C, s.K) &&
           (T * (s.C / 4) + 255) / 256 <= 0x7FFFFFFFll && (T * (s.K / 4) + 255) / 256 <= 0x7FFFFFFFll && (long long)s.K * s.C < 0x7FFFFFFFll;
}

void winograd_workspace(const ConvShape &s, size_t *u_bytes, size_t *v_bytes, size_t *m_bytes)
{
    const size_t T = (size_t)tile_count(s);
    *u_bytes = (size_t)16 * s.K * s.C * 2;
    *v_bytes = (size_t)16 * T * s.C * 2;
    *m_bytes = (size_t)16 * T * s.K * 4;
}

int winograd_fwd(const ConvShape &s, const void *x, const void *w, void *y, void *u, void *v, void *m, hipStream_t st,
                 const char **variant, const PostOp &post)
{
    const long long T = tile_count(s);
    const int TP = (s.P + 1) / 2, TQ = (s.Q + 1) / 2;
    hipLaunchKernelGGL(wino_filter_kernel, dim3((unsigned)((s.K * s.C + 255) / 256)), dim3(256), 0, st, (const bf16_t *)w, (bf16_t *)u, s.K, s.C);
    if (ok() != MXC_OK) return MXC_ERR_LAUNCH;
    hipLaunchKernelGGL(wino_input_kernel, dim3((unsigned)((T * (s.C / 4) + 255) / 256)), dim3(256), 0, st, (const bf16_t *)x, (bf16_t *)v, T,
                       TP, TQ, s.H, s.W, s.C, s.pad);
    if (ok() != MXC_OK) return MXC_ERR_LAUNCH;
    const char *gv = "";
    for (int xi = 0; xi < 16; ++xi) {
        const int rc = igemm_gemm_f32(T, s.C, s.K, (const bf16_t *)v + (size_t)xi * T * s.C, (const bf16_t *)u + (size_t)xi * s.K * s.C,
                                      (float *)m + (size_t)xi * T * s.K, st, &gv);
        if (rc != MXC_OK) return rc;
    }
    static thread_local char name[96];
    snprintf(name, sizeof(name), "winograd_f2x2_3x3+16x%s", gv);
    *variant = name;
    hipLaunchKernelGGL(wino_output_kernel, dim3((unsigned)((T * (s.K / 4) + 255) / 256)), dim3(256), 0, st, (const float *)m, (bf16_t *)y, T,
                       TP, TQ, s.P, s.Q, s.K, post.bias, post.relu);
    return ok();
}

}  // namespace mxc
