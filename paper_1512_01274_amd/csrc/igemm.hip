// bf16 implicit-GEMM convolution on the gfx950 matrix cores.
//
// One kernel family serves forward and backward-data.  The GEMM view is
//     Out[m][co] = sum_{t,ci} In[pixel(m) + tap(t)][ci] * Wm[co][t*Ci + ci]
// with m running over (image, output row, output column) of the launch's output grid, t over a
// TR x TS grid of filter taps, ci over input channels.  Both operands are contiguous along the
// reduction index (NHWC activations, filter rows of length T*Ci), which is the operand order the
// MFMA instructions want: every lane feeds 8 consecutive reduction elements of one row.
//
//   forward:        In = x,  Wm = w (KRSC),  pixel = (p*stride-pad, q*stride-pad), tap step +1
//   backward-data:  In = dy, Wm = per-phase re-packed filter [C][taps*K], one launch per residue
//                   class of (h+pad, v+pad) mod stride, tap step -1, strided output addressing.
//
// Tiling: a workgroup of 4 waves owns a BM x BN output tile; the reduction advances in steps of
// BK = 64 through a double-buffered LDS tile pair (A: BM x 64, B: BN x 64, 16-byte chunks XOR
// swizzled by row so that ds_read_b128 operand fetches are bank-conflict free).  Each wave
// accumulates a (BM/WR) x (BN/WC) sub-tile with v_mfma_f32_32x32x16_bf16 in fp32.
#include "mxc_internal.h"

namespace mxc {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BK = 64;           // reduction elements per LDS stage
constexpr int CHUNKS = BK / 8;   // 16-byte chunks per tile row

struct IgemmParams {
    const bf16_t *in;    // activations [N][Hi][Wi][Ci]
    const bf16_t *wm;    // filter matrix [Co][T*Ci]
    bf16_t *out;         // output tensor [N][Ho][Wo][Co]
    int N, Hi, Wi, Ci;
    int Co;
    int TR, TS, tstep;   // tap grid and direction (+1 or -1)
    int Mh, Mw;          // output grid of this launch (per image)
    int in_mul, in_off_h, in_off_w;     // input coordinate of tap 0: a*in_mul + in_off
    int Ho, Wo, out_mul, out_off_h, out_off_w;  // output coordinate: a*out_mul + out_off
    int m_tiles, n_tiles;
};

__device__ __forceinline__ uint4 ldg16(const bf16_t *p) { return *reinterpret_cast<const uint4 *>(p); }

template <int BM, int BN, int WR, int WC>
__global__ __launch_bounds__(64 * WR * WC) void igemm_kernel(const IgemmParams p)
{
    constexpr int NT = 64 * WR * WC;
    constexpr int WM = BM / WR, WN = BN / WC;     // wave tile
    constexpr int MI = WM / 32, NI = WN / 32;     // 32x32 MFMA blocks per wave
    constexpr int A_LD = BM * CHUNKS / NT;        // 16-byte loads per thread per stage
    constexpr int B_LD = BN * CHUNKS / NT;
    static_assert(BM * CHUNKS % NT == 0 && BN * CHUNKS % NT == 0, "tile/threads mismatch");
    static_assert(NT % CHUNKS == 0, "chunk column must be fixed per thread");

    __shared__ __attribute__((aligned(16))) bf16_t lds_a[2][BM * BK];
    __shared__ __attribute__((aligned(16))) bf16_t lds_b[2][BN * BK];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m = (wave / WC) * WM, wave_n = (wave % WC) * WN;

    // Workgroup -> tile.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs; give each
    // XCD a contiguous range of tiles, n-tile fastest, so that tiles sharing an activation tile meet
    // in one L2.
    const int total = p.m_tiles * p.n_tiles;
    const int per_xcd = (total + 7) / 8;
    int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;
    const int m0 = (logical / p.n_tiles) * BM, n0 = (logical % p.n_tiles) * BN;

    const long long M = (long long)p.N * p.Mh * p.Mw;
    const int T = p.TR * p.TS;
    const int Kd = T * p.Ci;
    const int KT = (Kd + BK - 1) / BK;

    // ---- per-thread load bookkeeping ------------------------------------------------------
    const int ld_col = tid % CHUNKS;          // chunk column (fixed), rows tid/CHUNKS + i*(NT/CHUNKS)
    const int ld_row0 = tid / CHUNKS;
    constexpr int ROW_STEP = NT / CHUNKS;

    long long a_base[A_LD];   // element offset of (n, base_h, base_w, 0); meaningless when !a_ok
    int a_h[A_LD], a_w[A_LD];
    bool a_ok[A_LD];
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const long long m = (long long)m0 + ld_row0 + i * ROW_STEP;
        a_ok[i] = m < M;
        const long long mm = a_ok[i] ? m : 0;
        const int b = (int)(mm % p.Mw);
        const long long t2 = mm / p.Mw;
        const int a = (int)(t2 % p.Mh);
        const int n = (int)(t2 / p.Mh);
        a_h[i] = a * p.in_mul + p.in_off_h;
        a_w[i] = b * p.in_mul + p.in_off_w;
        a_base[i] = (((long long)n * p.Hi + a_h[i]) * p.Wi + a_w[i]) * p.Ci;
    }
    long long b_base[B_LD];
    bool b_ok[B_LD];
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        const int co = n0 + ld_row0 + i * ROW_STEP;
        b_ok[i] = co < p.Co;
        b_base[i] = (long long)(b_ok[i] ? co : 0) * Kd;
    }
    // reduction position of this thread's chunk column: kd = kt*BK + ld_col*8 = tap*Ci + ci
    int kd = ld_col * 8;
    int ci = kd % p.Ci, tap = kd / p.Ci;
    int tr = p.TS > 0 ? tap / p.TS : 0, ts = p.TS > 0 ? tap % p.TS : 0;

    uint4 ra[A_LD], rb[B_LD];

    auto load_global = [&]() {
        const bool k_ok = kd < Kd;
        const int dh = tr * p.tstep, dv = ts * p.tstep;
        const long long tap_off = ((long long)dh * p.Wi + dv) * p.Ci + ci;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const bool ok = a_ok[i] && k_ok && (unsigned)(a_h[i] + dh) < (unsigned)p.Hi &&
                            (unsigned)(a_w[i] + dv) < (unsigned)p.Wi;
            ra[i] = ok ? ldg16(p.in + a_base[i] + tap_off) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) rb[i] = (b_ok[i] && k_ok) ? ldg16(p.wm + b_base[i] + kd) : make_uint4(0, 0, 0, 0);
        // advance to the next stage
        kd += BK;
        ci += BK;
        while (ci >= p.Ci) {
            ci -= p.Ci;
            if (++ts == p.TS) { ts = 0; ++tr; }
        }
    };

    auto store_lds = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const int row = ld_row0 + i * ROW_STEP;
            *reinterpret_cast<uint4 *>(&lds_a[buf][row * BK + ((ld_col ^ (row & 7)) << 3)]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            const int row = ld_row0 + i * ROW_STEP;
            *reinterpret_cast<uint4 *>(&lds_b[buf][row * BK + ((ld_col ^ (row & 7)) << 3)]) = rb[i];
        }
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int frag_row = lane & 31, frag_kg = lane >> 5;   // operand row and 8-element k group of this lane

    if (KT > 0) {
        load_global();
        store_lds(0);
    }
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_global();
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[MI], fb[NI];
            const int chunk = ks * 2 + frag_kg;
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const int row = wave_m + i * 32 + frag_row;
                fa[i] = *reinterpret_cast<const bf16x8 *>(&lds_a[buf][row * BK + ((chunk ^ (row & 7)) << 3)]);
            }
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int row = wave_n + j * 32 + frag_row;
                fb[j] = *reinterpret_cast<const bf16x8 *>(&lds_b[buf][row * BK + ((chunk ^ (row & 7)) << 3)]);
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_lds(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: fp32 -> bf16 (RNE), scatter to the output pixels -------------------------
    // accumulator element e of a 32x32 block: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const long long m = (long long)m0 + wave_m + i * 32 + 8 * (e >> 2) + 4 * frag_kg + (e & 3);
            if (m >= M) continue;
            const int b = (int)(m % p.Mw);
            const long long t2 = m / p.Mw;
            const int a = (int)(t2 % p.Mh);
            const int n = (int)(t2 / p.Mh);
            const long long pix = ((long long)n * p.Ho + (a * p.out_mul + p.out_off_h)) * p.Wo + (b * p.out_mul + p.out_off_w);
            bf16_t *orow = p.out + pix * p.Co;
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                const int co = n0 + wave_n + j * 32 + frag_row;
                if (co < p.Co) orow[co] = f32_to_bf16(acc[i][j][e]);
            }
        }
    }
}

template <int BM, int BN, int WR, int WC>
int launch(IgemmParams p, hipStream_t st)
{
    const long long M = (long long)p.N * p.Mh * p.Mw;
    const long long mt = (M + BM - 1) / BM;
    p.n_tiles = (p.Co + BN - 1) / BN;
    if (mt * p.n_tiles > 0x3FFFFFFFll) return MXC_ERR_SHAPE;
    p.m_tiles = (int)mt;
    const int total = p.m_tiles * p.n_tiles;
    const int grid = ((total + 7) / 8) * 8;
    hipLaunchKernelGGL((igemm_kernel<BM, BN, WR, WC>), dim3((unsigned)grid), dim3(64 * WR * WC), 0, st, p);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

// Re-pack the filter for backward-data.  For the residue class (ph, pw) of (h+pad, v+pad) mod
// stride the taps are r = ph + stride*j, s = pw + stride*i; its matrix is
//     wt[c][(j*TS + i)*K + k] = w[k][r][s][c]          (w in KRSC)
// and the classes are laid out one after another (sizes sum to K*R*S*C).
__global__ __launch_bounds__(256) void repack_bwd_data_filter_kernel(const bf16_t *__restrict__ w, bf16_t *__restrict__ wt,
                                                                     int K, int C, int R, int S, int stride)
{
    const int total = K * R * S * C;
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    // gid enumerates the destination: phase-major, then c, j, i, k
    int rem = gid, ph = 0, pw = 0, TR = 0, TS = 0;
    for (int a = 0; a < stride; ++a) {
        bool found = false;
        const int tr_a = a < R ? (R - a + stride - 1) / stride : 0;
        for (int b = 0; b < stride; ++b) {
            const int ts_b = b < S ? (S - b + stride - 1) / stride : 0;
            const int sz = C * tr_a * ts_b * K;
            if (rem < sz) { ph = a; pw = b; TR = tr_a; TS = ts_b; found = true; break; }
            rem -= sz;
        }
        if (found) break;
    }
    const int k = rem % K; rem /= K;
    const int i = rem % TS; rem /= TS;
    const int j = rem % TR; rem /= TR;
    const int c = rem;
    const int r = ph + stride * j, s = pw + stride * i;
    wt[gid] = w[(((size_t)k * R + r) * S + s) * C + c];
}

}  // namespace

bool igemm_fwd_supported(const ConvShape &s) { return s.C % 8 == 0; }

int igemm_fwd(const ConvShape &s, const void *x, const void *w, void *y, hipStream_t st, const char **variant)
{
    IgemmParams p{};
    p.in = (const bf16_t *)x; p.wm = (const bf16_t *)w; p.out = (bf16_t *)y;
    p.N = s.N; p.Hi = s.H; p.Wi = s.W; p.Ci = s.C; p.Co = s.K;
    p.TR = s.R; p.TS = s.S; p.tstep = 1;
    p.Mh = s.P; p.Mw = s.Q;
    p.in_mul = s.stride; p.in_off_h = -s.pad; p.in_off_w = -s.pad;
    p.Ho = s.P; p.Wo = s.Q; p.out_mul = 1; p.out_off_h = 0; p.out_off_w = 0;
    *variant = "igemm_128x128";
    return launch<128, 128, 2, 2>(p, st);
}

bool igemm_bwd_data_supported(const ConvShape &s) { return s.K % 8 == 0 && s.stride <= 4; }

size_t igemm_bwd_data_workspace(const ConvShape &s) { return (size_t)s.K * s.R * s.S * s.C * sizeof(bf16_t); }

int igemm_bwd_data(const ConvShape &s, const void *dy, const void *w, void *dx, void *wt, hipStream_t st,
                   const char **variant)
{
    const int total = s.K * s.R * s.S * s.C;
    hipLaunchKernelGGL(repack_bwd_data_filter_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       (const bf16_t *)w, (bf16_t *)wt, s.K, s.C, s.R, s.S, s.stride);
    if (hipGetLastError() != hipSuccess) return MXC_ERR_LAUNCH;
    size_t wt_off = 0;
    for (int ph = 0; ph < s.stride; ++ph) {
        for (int pw = 0; pw < s.stride; ++pw) {
            const int TR = ph < s.R ? (s.R - ph + s.stride - 1) / s.stride : 0;
            const int TS = pw < s.S ? (s.S - pw + s.stride - 1) / s.stride : 0;
            // output rows h = ph - pad + stride*hh >= 0, h < H
            const int hh0 = ph >= s.pad ? 0 : (s.pad - ph + s.stride - 1) / s.stride;
            const int vv0 = pw >= s.pad ? 0 : (s.pad - pw + s.stride - 1) / s.stride;
            const int h_first = ph - s.pad + s.stride * hh0, v_first = pw - s.pad + s.stride * vv0;
            const int Mh = h_first < s.H ? (s.H - 1 - h_first) / s.stride + 1 : 0;
            const int Mw = v_first < s.W ? (s.W - 1 - v_first) / s.stride + 1 : 0;
            IgemmParams p{};
            p.in = (const bf16_t *)dy; p.wm = (const bf16_t *)wt + wt_off; p.out = (bf16_t *)dx;
            p.N = s.N; p.Hi = s.P; p.Wi = s.Q; p.Ci = s.K; p.Co = s.C;
            p.TR = TR; p.TS = TS; p.tstep = -1;
            p.Mh = Mh; p.Mw = Mw;
            p.in_mul = 1; p.in_off_h = hh0; p.in_off_w = vv0;
            p.Ho = s.H; p.Wo = s.W; p.out_mul = s.stride; p.out_off_h = h_first; p.out_off_w = v_first;
            wt_off += (size_t)s.C * TR * TS * s.K;
            if (Mh <= 0 || Mw <= 0) continue;
            const int rc = launch<128, 128, 2, 2>(p, st);
            if (rc != MXC_OK) return rc;
        }
    }
    *variant = "igemm_128x128";
    return MXC_OK;
}

}  // namespace mxc
