// Operand re-packing for channel counts the MFMA kernels cannot gather directly.
//
// The MFMA kernels fetch 16-byte chunks (8 bf16) that must not straddle a filter tap.  Two
// re-packings make any channel count fit:
//   - channel padding: [rows][C] -> [rows][C8], C8 = C rounded up to 8, zeros in the new channels
//     (used when C % 8 != 0 and C > 4);
//   - small-C image packing (C <= 4, first layers): the image gets `pix` (4 or 8) channels per pixel
//     and an explicit zero border, so that for one filter row r the taps s = 0..S-1 of all channels
//     form ONE contiguous run of S*pix elements - the reduction then walks R long runs instead of
//     R*S*C scattered triples, and no bounds test can fail.  The filter is laid out to match:
//     [K][R][run], run = S*pix rounded up to 8, zeros where s >= S or c >= C.
// Pure data movement (bf16 bit patterns).
#include "mxc_internal.h"

namespace mxc {

namespace {

__global__ __launch_bounds__(256) void pad_channels_kernel(const bf16_t *__restrict__ src, uint4 *__restrict__ dst,
                                                           long long rows, int C, int C8)
{
    const int chunks = C8 >> 3;
    const long long total = rows * chunks;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const long long row = gid / chunks;
    const int c0 = (int)(gid % chunks) * 8;
    const bf16_t *s = src + row * C;
    uint32_t v[4] = {0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int c = c0 + j;
        const uint32_t e = c < C ? s[c] : 0u;
        v[j >> 1] |= e << ((j & 1) * 16);
    }
    dst[gid] = make_uint4(v[0], v[1], v[2], v[3]);
}

// xp[n][hp][wp][pix] = x[n][hp-pad][wp-pad][c] inside the image and for c < C, else 0.  One thread per 8 bytes.
__global__ __launch_bounds__(256) void smallc_pack_x_kernel(const bf16_t *__restrict__ x, uint2 *__restrict__ xp, int N, int C,
                                                            int H, int W, int pad, int Hp, int Wp, int pix)
{
    const int per_pix = pix >> 2;   // 8-byte pieces per pixel
    const long long total = (long long)N * Hp * Wp * per_pix;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const int piece = (int)(gid % per_pix);
    long long t = gid / per_pix;
    const int wp = (int)(t % Wp); t /= Wp;
    const int hp = (int)(t % Hp);
    const int n = (int)(t / Hp);
    const int h = hp - pad, w = wp - pad;
    uint32_t v[2] = {0, 0};
    if (piece == 0 && h >= 0 && h < H && w >= 0 && w < W) {
        const bf16_t *s = x + (((long long)n * H + h) * W + w) * C;
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (c < C) v[c >> 1] |= (uint32_t)s[c] << ((c & 1) * 16);
    }
    xp[gid] = make_uint2(v[0], v[1]);
}

// wp[k][r][s*pix + c] = w[k][r][s][c], zero elsewhere in the run
__global__ __launch_bounds__(256) void smallc_pack_w_kernel(const bf16_t *__restrict__ w, bf16_t *__restrict__ wp, int K, int C,
                                                            int R, int S, int pix, int run)
{
    const int total = K * R * run;
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const int e = gid % run;
    const int kr = gid / run;
    const int s = e / pix, c = e % pix;
    wp[gid] = (s < S && c < C) ? w[((size_t)kr * S + s) * C + c] : (bf16_t)0;
}

inline int ok() { return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH; }

}  // namespace

int pad_channels(const void *src, void *dst, long long rows, int C, hipStream_t st)
{
    const int C8 = (C + 7) / 8 * 8;
    const long long total = rows * (C8 / 8);
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return MXC_ERR_SHAPE;
    hipLaunchKernelGGL(pad_channels_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const bf16_t *)src, (uint4 *)dst, rows, C,
                       C8);
    return ok();
}

SmallCGeom smallc_geom(const ConvShape &s)
{
    SmallCGeom g;
    // window origins sit at pixel q*stride of the padded row: 16-byte aligned for every q only if
    // stride*pix is a multiple of 8
    g.pix = (s.stride % 2 == 0) ? 4 : 8;
    g.Hp = s.H + 2 * s.pad;
    g.Wp = (s.W + 2 * s.pad + 1) / 2 * 2;
    g.run = (s.S * g.pix + 7) / 8 * 8;
    return g;
}

int smallc_pack_x(const ConvShape &s, const void *x, void *xp, hipStream_t st)
{
    const SmallCGeom g = smallc_geom(s);
    const long long total = (long long)s.N * g.Hp * g.Wp * (g.pix / 4);
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return MXC_ERR_SHAPE;
    hipLaunchKernelGGL(smallc_pack_x_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const bf16_t *)x, (uint2 *)xp, s.N, s.C,
                       s.H, s.W, s.pad, g.Hp, g.Wp, g.pix);
    return ok();
}

int smallc_pack_w(const ConvShape &s, const void *w, void *wp, hipStream_t st)
{
    const SmallCGeom g = smallc_geom(s);
    const int total = s.K * s.R * g.run;
    hipLaunchKernelGGL(smallc_pack_w_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16_t *)w,
                       (bf16_t *)wp, s.K, s.C, s.R, s.S, g.pix, g.run);
    return ok();
}

}  // namespace mxc
