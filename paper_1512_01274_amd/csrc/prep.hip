// Operand re-packing for channel counts the MFMA kernels cannot gather directly.
//
// The MFMA kernels fetch 16-byte chunks (8 bf16) that must not straddle a filter tap.  Two
// re-packings make any channel count fit:
//   - channel padding: [rows][C] -> [rows][C8], C8 = C rounded up to 8, zeros in the new channels
//     (used when C % 8 != 0 and C > 4);
//   - space-to-depth (C <= 4, stride 2 or 4, first layers): stride x stride pixel blocks become the
//     channels of one pixel of a stride-1 problem, x2[n][h2][w2][(dh*s+dw)*Cq+c] with the zero border
//     folded in, filter likewise (zero taps beyond R,S); all three passes then run the ordinary
//     kernels on a stride-1 convolution with s*s*Cq channels;
//   - small-C image packing (C <= 4, stride 1): the image gets `pix` (4) channels per pixel
//     and an explicit zero border, so that for one filter row r the taps s = 0..S-1 of all channels
//     form ONE contiguous run of S*pix elements - the reduction then walks R long runs instead of
//     R*S*C scattered triples, and no bounds test can fail.  The filter is laid out to match:
//     [K][R][run], run = S*pix rounded up to 8, zeros where s >= S or c >= C.
// Pure data movement (bf16 bit patterns).
#include <type_traits>

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

// x2[n][h2][w2][(dh*s+dw)*Cq + c] = x[n][h2*s+dh-pad][w2*s+dw-pad][c] (0 outside the image or for c >= C).
// One thread per source pixel slot (n, h2, w2, dh, dw): Cq elements; consecutive threads write
// consecutive addresses and, within one dh, read consecutive addresses.
__global__ __launch_bounds__(256) void s2d_pack_x_kernel(const bf16_t *__restrict__ x, bf16_t *__restrict__ x2, int N, int C, int H,
                                                         int W, int pad, int s, int Cq, int H2, int W2)
{
    const int ss = s * s;
    const long long total = (long long)N * H2 * W2 * ss;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const int blk = (int)(gid % ss);
    long long t = gid / ss;
    const int w2 = (int)(t % W2); t /= W2;
    const int h2 = (int)(t % H2);
    const int n = (int)(t / H2);
    const int h = h2 * s + blk / s - pad, w = w2 * s + blk % s - pad;
    const bool in = h >= 0 && h < H && w >= 0 && w < W;
    const bf16_t *src = x + (((long long)n * H + h) * W + w) * C;
    bf16_t *dst = x2 + gid * Cq;
    for (int c = 0; c < Cq; ++c) dst[c] = (in && c < C) ? src[c] : (bf16_t)0;
}

// w2[k][r2][s2][(dh*s+dw)*Cq + c] = w[k][r2*s+dh][s2*s+dw][c], zero where r >= R, s >= S or c >= C
__global__ __launch_bounds__(256) void s2d_pack_w_kernel(const bf16_t *__restrict__ w, bf16_t *__restrict__ w2, int K, int C, int R,
                                                         int S, int s, int Cq, int C2, int R2, int S2)
{
    const int total = K * R2 * S2 * C2;
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const int e = gid % C2; int t = gid / C2;
    const int sb = t % S2; t /= S2;
    const int rb = t % R2;
    const int k = t / R2;
    const int blk = e / Cq, c = e % Cq;
    const int r = rb * s + blk / s, sc = sb * s + blk % s;
    w2[gid] = (c < C && r < R && sc < S) ? w[(((size_t)k * R + r) * S + sc) * C + c] : (bf16_t)0;
}

// dx[n][h][w][c] = dx2[n][(h+pad)/s][(w+pad)/s][(((h+pad)%s)*s + (w+pad)%s)*Cq + c]; 0 where no window reaches
__global__ __launch_bounds__(256) void s2d_unpack_dx_kernel(const bf16_t *__restrict__ dx2, bf16_t *__restrict__ dx, int N, int C,
                                                            int H, int W, int pad, int s, int Cq, int C2, int H2, int W2,
                                                            const bf16_t *__restrict__ mask)
{
    const long long total = (long long)N * H * W;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const int w = (int)(gid % W);
    long long t = gid / W;
    const int h = (int)(t % H);
    const int n = (int)(t / H);
    const int hp = h + pad, wp = w + pad;
    const int h2 = hp / s, w2 = wp / s;
    const bool in = h2 < H2 && w2 < W2;
    const bf16_t *src = dx2 + (((long long)n * H2 + h2) * W2 + w2) * C2 + ((hp % s) * s + wp % s) * Cq;
    bf16_t *d = dx + gid * C;
    for (int c = 0; c < C; ++c) d[c] = (in && (mask == nullptr || mask_keeps(mask + gid * C + c))) ? src[c] : (bf16_t)0;
}

// Fast space-to-depth copy for C == Cq when every run of s*C elements (one source row piece of a
// block) starts on a 4-byte boundary on both sides.  One thread per (n, h2, w2, dh), dh fastest: the
// four threads of a block touch one contiguous destination (pack) or source (unpack) pixel of x2.
// PACK:   x2 <- x, zeros outside the image.
// UNPACK: dx <- dx2 for pixels inside the image; blocks beyond the H2 x W2 grid (pixels no window
//         reaches) deliver zeros.  The grid covers ceil((H+pad)/s) x ceil((W+pad)/s) blocks.
template <bool PACK>
__global__ __launch_bounds__(256) void s2d_rows_kernel(const bf16_t *__restrict__ src, bf16_t *__restrict__ dst, int N, int C, int H,
                                                       int W, int pad, int s, int H2, int W2, int H2g, int W2g,
                                                       const bf16_t *__restrict__ mask)
{
    const long long total = (long long)N * H2g * W2g * s;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const int dh = (int)(gid % s);
    long long t = gid / s;
    const int w2 = (int)(t % W2g); t /= W2g;
    const int h2 = (int)(t % H2g);
    const int n = (int)(t / H2g);
    const int h = h2 * s + dh - pad, w0 = w2 * s - pad;
    const int run = s * C;
    const bool blk_ok = h2 < H2 && w2 < W2;                       // block exists in x2
    const long long img = ((long long)n * H + h) * W * C + (long long)w0 * C;          // element offset in x / dx
    const long long blk = ((((long long)n * H2 + h2) * W2 + w2) * s + dh) * run;      // element offset in x2 / dx2
    const bool row_ok = h >= 0 && h < H;
    const bool inside = row_ok && w0 >= 0 && w0 + s <= W;
    if (PACK) {
        if (!blk_ok) return;
        if (inside) {
            const uint32_t *a = reinterpret_cast<const uint32_t *>(src + img);
            uint32_t *b = reinterpret_cast<uint32_t *>(dst + blk);
            for (int i = 0; i < run / 2; ++i) b[i] = a[i];
        } else {
            for (int e = 0; e < run; ++e) {
                const int w = w0 + e / C;
                dst[blk + e] = (row_ok && w >= 0 && w < W) ? src[img + e] : (bf16_t)0;
            }
        }
    } else {
        if (!row_ok) return;
        if (inside && blk_ok) {
            const uint32_t *a = reinterpret_cast<const uint32_t *>(src + blk);
            uint32_t *b = reinterpret_cast<uint32_t *>(dst + img);
            const uint32_t *mk = reinterpret_cast<const uint32_t *>(mask + img);
            for (int i = 0; i < run / 2; ++i) b[i] = mask == nullptr ? a[i] : mask_bf16x2(a[i], mk[i]);
        } else {
            for (int e = 0; e < run; ++e) {
                const int w = w0 + e / C;
                if (w >= 0 && w < W)
                    dst[img + e] = (blk_ok && (mask == nullptr || mask_keeps(mask + img + e))) ? src[blk + e] : (bf16_t)0;
            }
        }
    }
}


// LDS-staged space-to-depth copies, same applicability as s2d_rows_kernel (C == Cq, every run of
// s*C elements dword-aligned on both sides).  One workgroup moves one row of blocks (n, h2): the s
// image rows and the x2 row are each contiguous in memory, so both sides are accessed with
// consecutive lanes on consecutive dwords (16 bytes per lane when V16: image rows 16-byte aligned),
// and the shuffle between the two orders happens in LDS at dword granularity.
//   image row dh, dword d  <->  x2 row dword ((w2*s + dh)*run + rem)/2,  with E = 2d + pad*C,
//   w2 = E / run, rem = E % run   (run = s*C elements).
template <bool V16>
__global__ __launch_bounds__(256) void s2d_stage_pack_kernel(const bf16_t *__restrict__ x, bf16_t *__restrict__ x2, int C, int H,
                                                             int W, int pad, int s, int H2, int W2)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t s2d_lds[];
    const int h2 = blockIdx.x % H2;
    const long long n = blockIdx.x / H2;
    const int row_dw = W * C / 2;                    // dwords per image row
    const int pitch = (row_dw + 3) & ~3;
    const int run_dw = s * C / 2;
    // all s image rows as one index space, up to NU loads in flight per thread before the first LDS write
    using T = std::conditional_t<V16, uint4, uint32_t>;
    const int per_row = V16 ? row_dw / 4 : row_dw;   // load units per image row
    const int lds_row = V16 ? pitch / 4 : pitch;
    const int total = s * per_row;
    constexpr int NU = 4;
    for (int base = threadIdx.x; base < total; base += 256 * NU) {
        T v[NU];
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int idx = base + u * 256;
            v[u] = T{};
            if (idx < total) {
                const int dh = idx / per_row, i = idx - dh * per_row;
                const int h = h2 * s + dh - pad;
                if (h >= 0 && h < H) v[u] = reinterpret_cast<const T *>(x + ((n * H + h) * W) * (long long)C)[i];
            }
        }
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int idx = base + u * 256;
            if (idx < total) {
                const int dh = idx / per_row, i = idx - dh * per_row;
                reinterpret_cast<T *>(s2d_lds)[dh * lds_row + i] = v[u];
            }
        }
    }
    __syncthreads();
    const int out_dw = W2 * s * run_dw;              // multiple of 4: s*s*C is a multiple of 8
    uint4 *dst = reinterpret_cast<uint4 *>(x2 + ((n * H2 + h2) * W2) * (long long)(s * s * C));
    const int shift = pad * C / 2;                   // dwords of left padding
    for (int o4 = threadIdx.x; o4 < out_dw / 4; o4 += 256) {
        int o = o4 * 4;
        int blk = o / run_dw, i = o - blk * run_dw;
        int w2 = blk / s, dh = blk - w2 * s;
        uint32_t v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int h = h2 * s + dh - pad;
            const int d = w2 * run_dw + i - shift;   // dword within the image row
            v[j] = (h >= 0 && h < H && d >= 0 && d < row_dw) ? s2d_lds[dh * pitch + d] : 0u;
            if (++i == run_dw) { i = 0; if (++dh == s) { dh = 0; ++w2; } }
        }
        dst[o4] = make_uint4(v[0], v[1], v[2], v[3]);
    }
}

// grid: N * H2g workgroups, H2g = ceil((H+pad)/s) rows of blocks cover every image row
template <bool V16>
__global__ __launch_bounds__(256) void s2d_stage_unpack_kernel(const bf16_t *__restrict__ dx2, bf16_t *__restrict__ dx, int C, int H,
                                                               int W, int pad, int s, int H2, int W2, int H2g,
                                                               const bf16_t *__restrict__ mask)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t s2d_lds[];
    const int h2 = blockIdx.x % H2g;
    const long long n = blockIdx.x / H2g;
    const int row_dw = W * C / 2;
    const int run_dw = s * C / 2;
    const int in_dw = W2 * s * run_dw;
    const bool have = h2 < H2;                       // beyond the last block row: zeros
    if (have) {
        const uint4 *src = reinterpret_cast<const uint4 *>(dx2 + ((n * H2 + h2) * W2) * (long long)(s * s * C));
        for (int i = threadIdx.x; i < in_dw / 4; i += 256) reinterpret_cast<uint4 *>(s2d_lds)[i] = src[i];
    }
    __syncthreads();
    const int shift = pad * C / 2;
    for (int dh = 0; dh < s; ++dh) {
        const int h = h2 * s + dh - pad;
        if (h < 0 || h >= H) continue;
        uint32_t *dst = reinterpret_cast<uint32_t *>(dx + ((n * H + h) * W) * (long long)C);
        const uint32_t *mk = reinterpret_cast<const uint32_t *>(mask + ((n * H + h) * W) * (long long)C);
        constexpr int V = V16 ? 4 : 1;
        for (int d0 = threadIdx.x * V; d0 < row_dw; d0 += 256 * V) {
            int E = d0 + shift;
            int w2 = E / run_dw, rem = E - w2 * run_dw;
            uint32_t v[V];
#pragma unroll
            for (int j = 0; j < V; ++j) {
                v[j] = (have && w2 < W2) ? s2d_lds[(w2 * s + dh) * run_dw + rem] : 0u;
                if (mask != nullptr) v[j] = mask_bf16x2(v[j], mk[d0 + j]);
                if (++rem == run_dw) { rem = 0; ++w2; }
            }
            if (V16) *reinterpret_cast<uint4 *>(dst + d0) = make_uint4(v[0], v[V > 1 ? 1 : 0], v[V > 2 ? 2 : 0], v[V > 3 ? 3 : 0]);
            else dst[d0] = v[0];
        }
    }
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
    // 4 channels per pixel: window origins are 8-byte aligned, which the 16-byte buffer loads accept
    g.pix = 4;
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

// every run of s*C elements starts 4-byte aligned in x and in x2 (and no channel padding)
static bool s2d_rows_aligned(const ConvShape &s, const S2DGeom &g)
{
    return g.Cq == s.C && (s.C % 2 == 0 || (s.W % 2 == 0 && s.pad % 2 == 0 && g.s % 2 == 0));
}

// both staging buffers (s image rows; one row of x2 blocks) fit the 64 KB of LDS a launch may ask for
static bool s2d_stage_fits(const ConvShape &s, const S2DGeom &g)
{
    const size_t img = (size_t)g.s * (((size_t)s.W * s.C / 2 + 3) & ~(size_t)3) * 4;
    const size_t blk = (size_t)g.W2 * g.C2 * 2;
    return img <= 65536 && blk <= 65536 && ((size_t)s.W * s.C) % 2 == 0;
}

S2DGeom s2d_geom(const ConvShape &s)
{
    S2DGeom g;
    g.s = s.stride;
    g.Cq = s.C;
    while ((g.s * g.s * g.Cq) % 8 != 0) ++g.Cq;
    g.C2 = g.s * g.s * g.Cq;
    g.R2 = (s.R + g.s - 1) / g.s;
    g.S2 = (s.S + g.s - 1) / g.s;
    g.H2 = s.P + g.R2 - 1;
    g.W2 = s.Q + g.S2 - 1;
    return g;
}

bool s2d_applicable(const ConvShape &s) { return s.C <= 4 && (s.stride == 2 || s.stride == 4); }

ConvShape s2d_shape(const ConvShape &s)
{
    const S2DGeom g = s2d_geom(s);
    return ConvShape{s.N, g.C2, g.H2, g.W2, s.K, g.R2, g.S2, 1, 0, s.P, s.Q};
}

int s2d_pack_x(const ConvShape &s, const void *x, void *x2, hipStream_t st)
{
    const S2DGeom g = s2d_geom(s);
    if (s2d_rows_aligned(s, g) && s2d_stage_fits(s, g) && (long long)s.N * g.H2 <= 0x7FFFFFFFll) {
        const bool v16 = ((long long)s.W * s.C * 2) % 16 == 0 && ((uintptr_t)x % 16) == 0;
        const size_t lds = (size_t)g.s * (((size_t)s.W * s.C / 2 + 3) & ~(size_t)3) * 4;
        const dim3 grid((unsigned)(s.N * g.H2));
        if (v16)
            hipLaunchKernelGGL(s2d_stage_pack_kernel<true>, grid, dim3(256), lds, st, (const bf16_t *)x, (bf16_t *)x2, s.C, s.H, s.W,
                               s.pad, g.s, g.H2, g.W2);
        else
            hipLaunchKernelGGL(s2d_stage_pack_kernel<false>, grid, dim3(256), lds, st, (const bf16_t *)x, (bf16_t *)x2, s.C, s.H, s.W,
                               s.pad, g.s, g.H2, g.W2);
        return ok();
    }
    if (s2d_rows_aligned(s, g)) {
        const long long n_thr = (long long)s.N * g.H2 * g.W2 * g.s;
        if ((n_thr + 255) / 256 > 0x7FFFFFFFll) return MXC_ERR_SHAPE;
        hipLaunchKernelGGL(s2d_rows_kernel<true>, dim3((unsigned)((n_thr + 255) / 256)), dim3(256), 0, st, (const bf16_t *)x,
                           (bf16_t *)x2, s.N, s.C, s.H, s.W, s.pad, g.s, g.H2, g.W2, g.H2, g.W2, (const bf16_t *)nullptr);
        return ok();
    }
    const long long total = (long long)s.N * g.H2 * g.W2 * g.s * g.s;
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return MXC_ERR_SHAPE;
    hipLaunchKernelGGL(s2d_pack_x_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const bf16_t *)x, (bf16_t *)x2, s.N, s.C, s.H,
                       s.W, s.pad, g.s, g.Cq, g.H2, g.W2);
    return ok();
}

int s2d_pack_w(const ConvShape &s, const void *w, void *w2, hipStream_t st)
{
    const S2DGeom g = s2d_geom(s);
    const int total = s.K * g.R2 * g.S2 * g.C2;
    hipLaunchKernelGGL(s2d_pack_w_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16_t *)w, (bf16_t *)w2,
                       s.K, s.C, s.R, s.S, g.s, g.Cq, g.C2, g.R2, g.S2);
    return ok();
}

int s2d_unpack_dx(const ConvShape &s, const void *dx2, void *dx, hipStream_t st, const void *mask)
{
    const S2DGeom g = s2d_geom(s);
    if (s2d_rows_aligned(s, g) && s2d_stage_fits(s, g) && (long long)s.N * ((s.H + s.pad + g.s - 1) / g.s) <= 0x7FFFFFFFll) {
        const int H2g = (s.H + s.pad + g.s - 1) / g.s;
        const bool v16 = ((long long)s.W * s.C * 2) % 16 == 0 && ((uintptr_t)dx % 16) == 0;
        const size_t lds = (size_t)g.W2 * g.C2 * 2;
        const dim3 grid((unsigned)(s.N * H2g));
        if (v16)
            hipLaunchKernelGGL(s2d_stage_unpack_kernel<true>, grid, dim3(256), lds, st, (const bf16_t *)dx2, (bf16_t *)dx, s.C, s.H,
                               s.W, s.pad, g.s, g.H2, g.W2, H2g, (const bf16_t *)mask);
        else
            hipLaunchKernelGGL(s2d_stage_unpack_kernel<false>, grid, dim3(256), lds, st, (const bf16_t *)dx2, (bf16_t *)dx, s.C, s.H,
                               s.W, s.pad, g.s, g.H2, g.W2, H2g, (const bf16_t *)mask);
        return ok();
    }
    if (s2d_rows_aligned(s, g)) {
        const int H2g = (s.H + s.pad + g.s - 1) / g.s, W2g = (s.W + s.pad + g.s - 1) / g.s;
        const long long n_thr = (long long)s.N * H2g * W2g * g.s;
        if ((n_thr + 255) / 256 > 0x7FFFFFFFll) return MXC_ERR_SHAPE;
        hipLaunchKernelGGL(s2d_rows_kernel<false>, dim3((unsigned)((n_thr + 255) / 256)), dim3(256), 0, st, (const bf16_t *)dx2,
                           (bf16_t *)dx, s.N, s.C, s.H, s.W, s.pad, g.s, g.H2, g.W2, H2g, W2g, (const bf16_t *)mask);
        return ok();
    }
    const long long total = (long long)s.N * s.H * s.W;
    const long long blocks = (total + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return MXC_ERR_SHAPE;
    hipLaunchKernelGGL(s2d_unpack_dx_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const bf16_t *)dx2, (bf16_t *)dx, s.N, s.C,
                       s.H, s.W, s.pad, g.s, g.Cq, g.C2, g.H2, g.W2, (const bf16_t *)mask);
    return ok();
}

}  // namespace mxc
