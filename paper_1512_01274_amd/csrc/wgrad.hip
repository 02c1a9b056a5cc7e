// bf16 backward-weight on the gfx950 matrix cores, split over the pixel reduction.
//
// GEMM view:  dw[k][col] = sum_m dy[m][k] * xcol[m][col],   col = (r*S + s)*C + c,
//             xcol[m][col] = x[n, p*stride-pad+r, q*stride-pad+s, c],   m = (n,p,q).
// The output matrix [K][R*S*C] is exactly dw in KRSC order.  The reduction index m is the slow
// axis of both NHWC operands, so tiles land in LDS as [pixel][channel] and the MFMA operands
// (8 consecutive reduction elements per lane) are fetched with the transposing LDS read
// ds_read_b64_tr_b16: within 16 lanes, lane j addresses 4 channels of pixel j/4 and receives
// the 4 pixels of channel j.
//
// Split reduction: workgroup (tile, z) reduces pixels [z*span, (z+1)*span) into an fp32 partial
// tile; a second kernel adds the partials of every tile in ascending z (fixed order, so results
// are bit-identical from run to run; no float atomics).
#include "mxc_internal.h"

namespace mxc {

namespace {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;

constexpr int BM = 128;   // k channels per tile
constexpr int BN = 128;   // filter columns (tap, c) per tile
constexpr int BP = 64;    // pixels per LDS stage
constexpr int NT = 256;
constexpr int ROW_CHUNKS = 16;            // 16-byte chunks per tile row (128 channels)
constexpr int ROWS_PER_PASS = NT / ROW_CHUNKS;   // 16
constexpr int LD = BP / ROWS_PER_PASS;           // 4 rows per thread per stage

struct WgradParams {
    const bf16_t *x;    // [N][H][W][C]
    const bf16_t *dy;   // [N][P][Q][K]
    float *partial;     // [splits][K][R*S*C]
    int N, C, H, W, K, R, S, stride, pad, P, Q;
    int k_tiles, n_tiles, splits;
    long long span;     // pixels per split (multiple of BP)
    // decomposition of a BP-pixel advance: BP = dq + Q*(dp + P*dn)
    int dq, dp, dn;
};

// physical position of 16-byte chunk `chunk` of tile row `row`
__device__ __forceinline__ int swz(int row, int chunk) { return row * (ROW_CHUNKS * 8) + ((chunk ^ ((row & 3) << 2)) << 3); }

__global__ __launch_bounds__(NT) void wgrad_kernel(const WgradParams p)
{
    __shared__ __attribute__((aligned(16))) bf16_t lds_a[2][BP * BM];   // dy tile  [pixel][k]
    __shared__ __attribute__((aligned(16))) bf16_t lds_b[2][BP * BN];   // x tile   [pixel][col]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = (wave >> 1) * 64, wave_n = (wave & 1) * 64;
    const int tile = blockIdx.x, z = blockIdx.y;
    const int k0 = (tile / p.n_tiles) * BM, n0 = (tile % p.n_tiles) * BN;
    const int RSC = p.R * p.S * p.C;
    const long long M = (long long)p.N * p.P * p.Q;
    const long long m_begin = (long long)z * p.span;
    long long m_end = m_begin + p.span;
    if (m_end > M) m_end = M;
    const int KT = m_end > m_begin ? (int)((m_end - m_begin + BP - 1) / BP) : 0;

    // ---- load bookkeeping: this thread owns chunk column ld_col of rows ld_row0 + 16*i ----
    const int ld_col = tid % ROW_CHUNKS, ld_row0 = tid / ROW_CHUNKS;
    const int kch = k0 + ld_col * 8;                 // dy channel of the chunk
    const bool a_col_ok = kch < p.K;
    const int col = n0 + ld_col * 8;                 // filter column of the chunk
    const bool b_col_ok = col < RSC;
    const int tap = b_col_ok ? col / p.C : 0, cc = b_col_ok ? col % p.C : 0;
    const int fr = tap / p.S, fs = tap % p.S;

    int pn[LD], pp[LD], pq[LD];
#pragma unroll
    for (int i = 0; i < LD; ++i) {
        const long long m = m_begin + ld_row0 + i * ROWS_PER_PASS;
        pq[i] = (int)(m % p.Q);
        const long long t = m / p.Q;
        pp[i] = (int)(t % p.P);
        pn[i] = (int)(t / p.P);
    }
    long long m_row = m_begin + ld_row0;   // pixel index of row i is m_row + 16*i

    uint4 ra[LD], rb[LD];
    auto load_global = [&]() {
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const long long m = m_row + i * ROWS_PER_PASS;
            const bool row_ok = m < m_end;
            ra[i] = (row_ok && a_col_ok) ? *reinterpret_cast<const uint4 *>(p.dy + m * p.K + kch) : make_uint4(0, 0, 0, 0);
            const int h = pp[i] * p.stride - p.pad + fr, v = pq[i] * p.stride - p.pad + fs;
            const bool ok = row_ok && b_col_ok && (unsigned)h < (unsigned)p.H && (unsigned)v < (unsigned)p.W;
            rb[i] = ok ? *reinterpret_cast<const uint4 *>(p.x + (((long long)pn[i] * p.H + h) * p.W + v) * p.C + cc)
                       : make_uint4(0, 0, 0, 0);
            // advance this row by BP pixels
            int q = pq[i] + p.dq;
            const int cq = q >= p.Q;
            q -= cq ? p.Q : 0;
            int pr = pp[i] + p.dp + cq;
            const int cp = pr >= p.P;
            pr -= cp ? p.P : 0;
            pq[i] = q; pp[i] = pr; pn[i] += p.dn + cp;
        }
        m_row += BP;
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int row = ld_row0 + i * ROWS_PER_PASS;
            *reinterpret_cast<uint4 *>(&lds_a[buf][swz(row, ld_col)]) = ra[i];
            *reinterpret_cast<uint4 *>(&lds_b[buf][swz(row, ld_col)]) = rb[i];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // transposing-read geometry: 16-lane group g, lane j within it
    const int g = lane >> 4, j16 = lane & 15;
    const int tr_row = (g >> 1) * 8 + (j16 >> 2);        // pixel row within a 16-pixel k-step (second read: +4)
    const int tr_ch = (g & 1) * 16 + (j16 & 3) * 4;      // channel within a 32-channel block

    auto frag = [&](const bf16_t *tile, int ch_base, int ks) -> bf16x8 {
        const int row = ks * 16 + tr_row;
        const int ch = ch_base + tr_ch;
        const bf16_t *p0 = tile + swz(row, ch >> 3) + (ch & 7);
        const bf16_t *p1 = tile + swz(row + 4, ch >> 3) + (ch & 7);
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)p0);
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)p1);
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    if (KT > 0) {
        load_global();
        store_lds(0);
    }
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_global();
#pragma unroll
        for (int ks = 0; ks < BP / 16; ++ks) {
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) fa[i] = frag(lds_a[buf], wave_m + i * 32, ks);
#pragma unroll
            for (int j = 0; j < 2; ++j) fb[j] = frag(lds_b[buf], wave_n + j * 32, ks);
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- fp32 partial tile -> workspace ------------------------------------------------------
    float *out = p.partial + (size_t)z * p.K * RSC;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int k = k0 + wave_m + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            if (k >= p.K) continue;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int c = n0 + wave_n + j * 32 + (lane & 31);
                if (c < RSC) out[(size_t)k * RSC + c] = acc[i][j][e];
            }
        }
}

// dw[i] = partial[0][i] + partial[1][i] + ... (ascending split order)
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float *__restrict__ partial, float *__restrict__ dw,
                                                           int total, int splits)
{
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    float acc = partial[gid];
    for (int zz = 1; zz < splits; ++zz) acc += partial[(size_t)zz * total + gid];
    dw[gid] = acc;
}

}  // namespace

bool wgrad_supported(const ConvShape &s) { return s.C % 8 == 0 && s.K % 8 == 0; }

int wgrad_splits(const ConvShape &s)
{
    const long long M = (long long)s.N * s.P * s.Q;
    const long long tiles = (long long)((s.K + BM - 1) / BM) * ((s.R * s.S * s.C + BN - 1) / BN);
    long long splits = (1024 + tiles - 1) / tiles;          // aim for ~4 workgroups per CU
    const long long max_by_work = (M + 4 * BP - 1) / (4 * BP);  // at least 4 stages per split
    if (splits > max_by_work) splits = max_by_work;
    if (splits > 1024) splits = 1024;
    if (splits < 1) splits = 1;
    return (int)splits;
}

size_t wgrad_workspace(const ConvShape &s)
{
    return (size_t)wgrad_splits(s) * s.K * s.R * s.S * s.C * sizeof(float);
}

int wgrad(const ConvShape &s, const void *x, const void *dy, float *dw, float *partial, hipStream_t st,
          const char **variant)
{
    WgradParams p{};
    p.x = (const bf16_t *)x; p.dy = (const bf16_t *)dy; p.partial = partial;
    p.N = s.N; p.C = s.C; p.H = s.H; p.W = s.W; p.K = s.K; p.R = s.R; p.S = s.S;
    p.stride = s.stride; p.pad = s.pad; p.P = s.P; p.Q = s.Q;
    p.k_tiles = (s.K + BM - 1) / BM;
    p.n_tiles = (s.R * s.S * s.C + BN - 1) / BN;
    p.splits = wgrad_splits(s);
    const long long M = (long long)s.N * s.P * s.Q;
    long long span = (M + p.splits - 1) / p.splits;
    span = (span + BP - 1) / BP * BP;
    p.span = span;
    p.dq = BP % s.Q;
    const int rows = BP / s.Q;
    p.dp = rows % s.P;
    p.dn = rows / s.P;
    const long long tiles = (long long)p.k_tiles * p.n_tiles;
    if (tiles > 0x7FFFFFFFll || p.splits > 65535) return MXC_ERR_SHAPE;
    hipLaunchKernelGGL(wgrad_kernel, dim3((unsigned)tiles, (unsigned)p.splits), dim3(NT), 0, st, p);
    if (hipGetLastError() != hipSuccess) return MXC_ERR_LAUNCH;
    const int total = s.K * s.R * s.S * s.C;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, partial, dw, total,
                       p.splits);
    *variant = "wgrad_128x128_splitk";
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

}  // namespace mxc
