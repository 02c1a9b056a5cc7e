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

constexpr int BK = 64;           // reduction elements per LDS stage (one 128-byte tile row)

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
    int linear_out;      // output pixel index == m (forward, and stride-1 backward-data)
    int M;               // N*Mh*Mw (< 2^31, checked by the launcher)
    int m_tiles, n_tiles;
};

// 16 bytes of zeros in global memory: the source of every tile chunk that lies in the padding,
// beyond the tensor or beyond the reduction length (direct-to-LDS loads cannot be predicated to
// write zeros, so such lanes are pointed here instead).
__device__ const uint4 g_zero_chunk[1] = {};

typedef __attribute__((address_space(3))) void *lds_vptr;
typedef const __attribute__((address_space(1))) void *glb_vptr;

// One wave-wide direct global->LDS transfer: lane l's 16 bytes land at lds_base + 16*l.
__device__ __forceinline__ void load16_to_lds(const bf16_t *src, bf16_t *lds_base_uniform)
{
    __builtin_amdgcn_global_load_lds((glb_vptr)src, (lds_vptr)lds_base_uniform, 16, 0, 0);
}

// Tile rows are 128 bytes (8 chunks).  Chunk c of row r is stored at chunk position c ^ swz(r):
// any 16 consecutive rows at one logical chunk then cover all 64 LDS banks exactly once.
__device__ __forceinline__ int swz(int row) { return (row >> 1) & 7; }

template <int BM, int BN, int WR, int WC>
__global__ __launch_bounds__(64 * WR * WC) void igemm_kernel(const IgemmParams p)
{
    constexpr int NW = WR * WC;
    constexpr int WM = BM / WR, WN = BN / WC;     // wave tile
    constexpr int MI = WM / 32, NI = WN / 32;     // 32x32 MFMA blocks per wave
    constexpr int A_LD = BM / 8 / NW;             // wave-wide loads (8 tile rows each) per wave per stage
    constexpr int B_LD = BN / 8 / NW;
    static_assert(NW % 2 == 0 && BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile/wave mismatch");

    __shared__ __attribute__((aligned(1024))) bf16_t lds_a[2][BM * BK];
    __shared__ __attribute__((aligned(1024))) bf16_t lds_b[2][BN * BK];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m = (wave / WC) * WM, wave_n = (wave % WC) * WN;

    // Workgroup -> tile.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs; give each
    // XCD a contiguous range of tiles, n-tile fastest, so that tiles sharing an activation tile meet
    // in one L2.
    const int total = p.m_tiles * p.n_tiles;
    const int per_xcd = (total + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total) return;
    const int m0 = (logical / p.n_tiles) * BM, n0 = (logical % p.n_tiles) * BN;

    const int T = p.TR * p.TS;
    const int Kd = T * p.Ci;
    const int KT = (Kd + BK - 1) / BK;

    // ---- load bookkeeping --------------------------------------------------------------------
    // Wave-wide load number i (of BM/8 for A) fills tile rows 8i..8i+7: lane l -> row 8i + l/8,
    // chunk position l%8.  This wave issues i = wave, wave+NW, ...; NW is even, so swz(row) and
    // with it the logical chunk (the reduction offset) a lane fetches is the same for all of them.
    const int ld_sub = lane >> 3;                                    // row within the 8-row group
    const int ld_chunk = (lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7);   // logical chunk fetched

    int a_off[A_LD];     // element offset of (n, base_h, base_w, 0) / 8   (may be negative)
    int a_hw[A_LD];      // base_h in the low 16 bits, base_w in the high 16 (both signed); row invalid: h = -32768
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int m = m0 + 8 * (wave + NW * i) + ld_sub;
        if (m < p.M) {
            const unsigned b = (unsigned)m % (unsigned)p.Mw, t2 = (unsigned)m / (unsigned)p.Mw;
            const unsigned a = t2 % (unsigned)p.Mh, n = t2 / (unsigned)p.Mh;
            const int h = (int)a * p.in_mul + p.in_off_h, w = (int)b * p.in_mul + p.in_off_w;
            a_off[i] = (int)((((long long)n * p.Hi + h) * p.Wi + w) * (p.Ci >> 3));
            a_hw[i] = (h & 0xFFFF) | (w << 16);
        } else {
            a_off[i] = 0;
            a_hw[i] = 0x8000;   // h = -32768: never inside the image
        }
    }
    // reduction position of this lane's chunk: kd = kt*BK + ld_chunk*8 = tap*Ci + ci
    int kd = ld_chunk * 8;
    int ci = kd % p.Ci;
    const int tap0 = kd / p.Ci;
    int tr = p.TS > 0 ? tap0 / p.TS : 0, ts = p.TS > 0 ? tap0 % p.TS : 0;
    const bf16_t *zero = reinterpret_cast<const bf16_t *>(g_zero_chunk);
    const int b_row0 = n0 + 8 * wave + ld_sub;    // filter row of load 0; load i: + 8*NW*i

    auto issue_loads = [&](int buf) {
        const bool k_ok = kd < Kd;
        const int dh = tr * p.tstep, dv = ts * p.tstep;
        const int tap_off = ((dh * p.Wi + dv) * p.Ci + ci) >> 3;
#pragma unroll
        for (int i = 0; i < A_LD; ++i) {
            const int h = (int)(short)(a_hw[i] & 0xFFFF) + dh, w = (a_hw[i] >> 16) + dv;
            const bool ok = k_ok && (unsigned)h < (unsigned)p.Hi && (unsigned)w < (unsigned)p.Wi;
            const bf16_t *src = ok ? p.in + ((long long)(a_off[i] + tap_off) << 3) : zero;
            load16_to_lds(src, &lds_a[buf][(wave + NW * i) * 8 * BK]);
        }
#pragma unroll
        for (int i = 0; i < B_LD; ++i) {
            const int co = b_row0 + 8 * NW * i;
            const bf16_t *src = (k_ok && co < p.Co) ? p.wm + ((long long)co * Kd + kd) : zero;
            load16_to_lds(src, &lds_b[buf][(wave + NW * i) * 8 * BK]);
        }
        kd += BK;
        ci += BK;
        while (ci >= p.Ci) {
            ci -= p.Ci;
            if (++ts == p.TS) { ts = 0; ++tr; }
        }
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // operand fetch: lane -> tile row (lane%32) of a 32-row block, 8-element group lane/32 of a 16-wide k step
    const int frag_row = lane & 31, frag_kg = lane >> 5;
    const int frag_swz = swz(frag_row);            // block bases are multiples of 32 rows: swz(row) == swz(frag_row)

    if (KT > 0) issue_loads(0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) issue_loads(buf ^ 1);
        const bf16_t *ta = &lds_a[buf][(wave_m + frag_row) * BK];
        const bf16_t *tb = &lds_b[buf][(wave_n + frag_row) * BK];
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[MI], fb[NI];
            const int pos = ((ks * 2 + frag_kg) ^ frag_swz) << 3;
#pragma unroll
            for (int i = 0; i < MI; ++i) fa[i] = *reinterpret_cast<const bf16x8 *>(ta + i * 32 * BK + pos);
#pragma unroll
            for (int j = 0; j < NI; ++j) fb[j] = *reinterpret_cast<const bf16x8 *>(tb + j * 32 * BK + pos);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }

    // ---- epilogue: fp32 -> bf16 (RNE), scatter to the output pixels -------------------------
    // accumulator element e of a 32x32 block: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int m = m0 + wave_m + i * 32 + 8 * (e >> 2) + 4 * frag_kg + (e & 3);
            if (m >= p.M) continue;
            long long pix = m;
            if (!p.linear_out) {
                const unsigned b = (unsigned)m % (unsigned)p.Mw, t2 = (unsigned)m / (unsigned)p.Mw;
                const unsigned a = t2 % (unsigned)p.Mh, n = t2 / (unsigned)p.Mh;
                pix = ((long long)n * p.Ho + ((int)a * p.out_mul + p.out_off_h)) * p.Wo + ((int)b * p.out_mul + p.out_off_w);
            }
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
    p.M = (int)M;
    p.m_tiles = (int)mt;
    p.linear_out = (p.out_mul == 1 && p.out_off_h == 0 && p.out_off_w == 0 && p.Mh == p.Ho && p.Mw == p.Wo) ? 1 : 0;
    const int total = p.m_tiles * p.n_tiles;
    const int grid = ((total + 7) / 8) * 8;
    hipLaunchKernelGGL((igemm_kernel<BM, BN, WR, WC>), dim3((unsigned)grid), dim3(64 * WR * WC), 0, st, p);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

// The kernel addresses activations with 32-bit offsets in units of 8 elements and packs tile-row
// coordinates into 16 bits.
bool igemm_dims_ok(long long in_elems, long long M, int Hi, int Wi, int span)
{
    return in_elems / 8 < 0x7FFFFFFFll && M < 0x7FFFFFFFll && Hi + span < 32000 && Wi + span < 32000;
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

bool igemm_fwd_supported(const ConvShape &s)
{
    return s.C % 8 == 0 && igemm_dims_ok((long long)s.N * s.H * s.W * s.C, (long long)s.N * s.P * s.Q, s.H, s.W,
                                         s.pad + s.R + s.S + s.stride);
}

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

bool igemm_bwd_data_supported(const ConvShape &s)
{
    return s.K % 8 == 0 && s.stride <= 4 &&
           igemm_dims_ok((long long)s.N * s.P * s.Q * s.K, (long long)s.N * s.H * s.W, s.P, s.Q, s.pad + s.R + s.S + s.stride);
}

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
