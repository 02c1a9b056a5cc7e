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
// Pipeline: a ring of NS LDS stages of BP pixels each, filled by direct global->LDS buffer loads
// (out-of-range lanes deposit zeros: padding, ragged edges, the tail of a split) issued NS stages
// ahead; address generation and operand fetches are interleaved between the MFMAs.
//
// Split reduction: workgroup (tile, z) reduces pixels [z*span, (z+1)*span) into an fp32 partial
// tile; a second kernel adds the partials of every element in a fixed order (lane groups of a wave take
// interleaved splits and exchange their sums with wave-level shuffles), so results are bit-identical from
// run to run; no float atomics.
#include <stdlib.h>
#include <string.h>

#include <type_traits>

#include "mxc_internal.h"

namespace mxc {

namespace {

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;
typedef __attribute__((address_space(3))) void *lds_vptr;
typedef short s16x2 __attribute__((ext_vector_type(2)));

constexpr unsigned OOB = 0x80000000u;   // a buffer offset no operand reaches: the load returns zeros

struct WgradParams {
    const bf16_t *x;    // [N][H][W][pix]
    const bf16_t *dy;   // [N][P][Q][K]
    float *partial;     // [splits][K][ncols]
    int N, H, W, pix;   // x geometry: pix elements per pixel in memory
    int K, P, Q, stride, pad;
    int TS, run, ncols; // filter columns: col = tap*run + e, tap = fr*TS + fs, e = offset in the tap's contiguous run
    int n_tiles, splits, tiles, n_wg;
    int span;           // pixels per split (multiple of the stage size)
    int M;              // N*P*Q
    int dq, dp, dn;     // decomposition of a one-stage pixel advance: BP = dq + Q*(dp + P*dn)
    unsigned x_bytes, dy_bytes;
};

template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ void wait_lgkmcnt0() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void pin() { __builtin_amdgcn_sched_barrier(0); }
// Workgroup barrier of the ring: the bare instruction, with the counters it needs waited for by hand just before
// it (a __syncthreads() would add fences the ring does not need).
__device__ __forceinline__ void ring_barrier() { pin(); __builtin_amdgcn_s_barrier(); pin(); }

template <int I> using IC = std::integral_constant<int, I>;
template <class F, int... I> __device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) { (f(IC<I>{}), ...); }
template <int N, class F> __device__ __forceinline__ void static_for(F &&f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

// XOR applied to the chunk index of tile row `row` (RC chunks of 16 bytes per row) so that the four
// pixel rows touched by one transposing read fall into different banks.
template <int RC> __device__ __forceinline__ int row_swz(int row)
{
    if constexpr (RC >= 16) return (row & 3) << 2;
    else if constexpr (RC == 8) return ((row >> 1) & 1) << 2;
    else return 0;
}

// BMT k-channels x BNT filter columns per tile, BP pixels per stage, NS stages, WR x WC waves.
template <int BMT, int BNT, int BP, int NS, int WR, int WC>
__global__ __launch_bounds__(64 * WR * WC, (WR * WC == 4 && NS * BP * (BMT + BNT) * 2 <= 80 * 1024) ? 2 : 1) void wgrad_kernel(
    const WgradParams p)
{
    constexpr int NW = WR * WC;
    constexpr int WM = BMT / WR, WN = BNT / WC;
    constexpr int MI = WM / 32, NI = WN / 32, NMF = MI * NI;
    constexpr int RCA = BMT / 8, RCB = BNT / 8;           // 16-byte chunks per tile row
    constexpr int RPLA = 64 / RCA, RPLB = 64 / RCB;       // pixel rows per wave-wide load
    constexpr int A_LD = BP / RPLA / NW, B_LD = BP / RPLB / NW;
    constexpr int L = A_LD + B_LD;
    constexpr int KS = BP / 16;
    static_assert(NS >= 2 && NS <= 4 && KS % 2 == 0 && NW % 2 == 0, "config");
    static_assert(BP % (RPLA * NW) == 0 && BP % (RPLB * NW) == 0 && RCA <= 32 && RCB <= 32 && RCA >= 4 && RCB >= 4, "tile/wave mismatch");
    static_assert(L * (NS - 1) < 64, "vmcnt range");

    constexpr int SZA = BP * BMT, SZB = BP * BNT;
    __shared__ __attribute__((aligned(1024))) bf16_t sa0[SZA];
    __shared__ __attribute__((aligned(1024))) bf16_t sa1[SZA];
    __shared__ __attribute__((aligned(1024))) bf16_t sa2[NS > 2 ? SZA : 8];
    __shared__ __attribute__((aligned(1024))) bf16_t sa3[NS > 3 ? SZA : 8];
    __shared__ __attribute__((aligned(1024))) bf16_t sb0[SZB];
    __shared__ __attribute__((aligned(1024))) bf16_t sb1[SZB];
    __shared__ __attribute__((aligned(1024))) bf16_t sb2[NS > 2 ? SZB : 8];
    __shared__ __attribute__((aligned(1024))) bf16_t sb3[NS > 3 ? SZB : 8];
    auto stage_a = [&](auto s) __attribute__((always_inline)) -> bf16_t * {
        constexpr int S = decltype(s)::value;
        if constexpr (S == 0) return sa0; else if constexpr (S == 1) return sa1; else if constexpr (S == 2) return sa2; else return sa3;
    };
    auto stage_b = [&](auto s) __attribute__((always_inline)) -> bf16_t * {
        constexpr int S = decltype(s)::value;
        if constexpr (S == 0) return sb0; else if constexpr (S == 1) return sb1; else if constexpr (S == 2) return sb2; else return sb3;
    };

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = (wave / WC) * WM, wave_n = (wave % WC) * WN;
    // Workgroup -> (split z, tile).  Consecutive workgroup ids go round-robin to the 8 XCDs; give each
    // XCD a contiguous range with the tile index fastest, so the tiles that reduce the same pixel
    // range (and read the same dy and x rows) share one L2.
    const int total_wg = p.n_wg;
    const int per_xcd = (total_wg + 7) / 8;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (logical >= total_wg) return;
    const int tile = logical % p.tiles, z = logical / p.tiles;
    const int k0 = (tile / p.n_tiles) * BMT, n0 = (tile % p.n_tiles) * BNT;
    const int RSC = p.ncols;
    const int m_begin = z * p.span;
    const int m_end = min(m_begin + p.span, p.M);
    const int KT = m_end > m_begin ? (m_end - m_begin + BP - 1) / BP : 0;

    const buf_rsrc_t rs_x = make_buf_rsrc(p.x, p.x_bytes);
    const buf_rsrc_t rs_dy = make_buf_rsrc(p.dy, p.dy_bytes);

    // ---- A side (dy): lane -> pixel row RPLA*i + lane/RCA of the stage, k-channel chunk fixed -------
    const int la_sub = lane / RCA;
    const int la_chunk = (lane % RCA) ^ row_swz<RCA>(RPLA * wave + la_sub);   // RPLA*NW*j never changes the swizzle
    const int kch = k0 + la_chunk * 8;
    int a_m[A_LD];                       // pixel index of this lane's row in the current stage
    unsigned a_col = kch < p.K ? (unsigned)kch * 2u : OOB;
#pragma unroll
    for (int i = 0; i < A_LD; ++i) a_m[i] = m_begin + RPLA * (wave + NW * i) + la_sub;

    // ---- B side (x gather): filter column chunk fixed per lane -> fixed tap (r,s) and channel ------
    const int lb_sub = lane / RCB;
    const int lb_chunk = (lane % RCB) ^ row_swz<RCB>(RPLB * wave + lb_sub);
    const int col = n0 + lb_chunk * 8;
    const bool col_ok = col < RSC;
    const int tap = col_ok ? col / p.run : 0, cc = col_ok ? col % p.run : 0;
    const int fr = tap / p.TS, fs = tap % p.TS;
    const int tap_off = col_ok ? ((fr * p.W + fs) * p.pix + cc) * 2 : 0;   // bytes, relative to the window origin
    // window origin (p*stride-pad, q*stride-pad) of each row, its byte offset, and (n,p,q) to advance it
    int b_n[B_LD], b_p[B_LD], b_q[B_LD], b_m[B_LD];
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        const int m = m_begin + RPLB * (wave + NW * i) + lb_sub;
        b_m[i] = m;
        b_q[i] = (int)((unsigned)m % (unsigned)p.Q);
        const unsigned t = (unsigned)m / (unsigned)p.Q;
        b_p[i] = (int)(t % (unsigned)p.P);
        b_n[i] = (int)(t / (unsigned)p.P);
    }
    const int lim_hw = ((p.H - 1) & 0xFFFF) | ((p.W - 1) << 16);
    const int tap_hw = ((fr - p.pad) & 0xFFFF) | ((fs - p.pad) << 16);

    unsigned va[A_LD], vb[B_LD];
    // address tasks: 0..A_LD-1 = dy rows, A_LD..A_LD+B_LD-1 = x rows (each also advances its row by one stage)
    auto addr_task = [&](auto t) __attribute__((always_inline)) {
        constexpr int Tk = decltype(t)::value;
        if constexpr (Tk < A_LD) {
            va[Tk] = a_m[Tk] < m_end ? (unsigned)a_m[Tk] * (unsigned)(p.K * 2) + a_col : OOB;
            a_m[Tk] += BP;
        } else {
            constexpr int i = Tk - A_LD;
            const int h0 = b_p[i] * p.stride, w0 = b_q[i] * p.stride;
            const s16x2 hw = __builtin_bit_cast(s16x2, (h0 & 0xFFFF) | (w0 << 16)) + __builtin_bit_cast(s16x2, tap_hw);
            const s16x2 d = __builtin_bit_cast(s16x2, lim_hw) - hw;
            const int bad = (__builtin_bit_cast(int, hw) | __builtin_bit_cast(int, d)) & (int)0x80008000;
            const int org = ((b_n[i] * p.H + h0 - p.pad) * p.W + (w0 - p.pad)) * (p.pix * 2);
            vb[i] = (bad == 0 && b_m[i] < m_end && col_ok) ? (unsigned)(org + tap_off) : OOB;
            // advance by BP pixels
            b_m[i] += BP;
            int q = b_q[i] + p.dq;
            const int cq = q >= p.Q ? 1 : 0;
            q -= cq ? p.Q : 0;
            int pr = b_p[i] + p.dp + cq;
            const int cp = pr >= p.P ? 1 : 0;
            pr -= cp ? p.P : 0;
            b_q[i] = q; b_p[i] = pr; b_n[i] += p.dn + cp;
        }
    };
    auto load_task = [&](auto t, bf16_t *dst_a, bf16_t *dst_b) __attribute__((always_inline)) {
        constexpr int Tk = decltype(t)::value;
        if constexpr (Tk < A_LD) lds_dma16(rs_dy, va[Tk], dst_a + (wave + NW * Tk) * RPLA * BMT);
        else lds_dma16(rs_x, vb[Tk - A_LD], dst_b + (wave + NW * (Tk - A_LD)) * RPLB * BNT);
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // transposing-read geometry: 16-lane group g, lane j within it.  One read: 4 pixel rows x 16 channels.
    const int g = lane >> 4, j16 = lane & 15;
    const int tr_row = (g >> 1) * 8 + (j16 >> 2);        // pixel row within a 16-pixel k-step (second read: +4)
    const int tr_ch = (g & 1) * 16 + (j16 & 3) * 4;      // channel within a 32-channel block
    // element offsets of the two reads within a 16-pixel k-step, per operand, for channel block 0
    auto tr_off = [&](auto rc, int ch_base, int row) __attribute__((always_inline)) {
        constexpr int RC = decltype(rc)::value;
        const int ch = ch_base + tr_ch;
        return row * (RC * 8) + ((((ch >> 3) ^ row_swz<RC>(row))) << 3) + (ch & 7);
    };
    int offa_lo[MI], offa_hi[MI], offb_lo[NI], offb_hi[NI];
#pragma unroll
    for (int i = 0; i < MI; ++i) { offa_lo[i] = tr_off(IC<RCA>{}, wave_m + i * 32, tr_row); offa_hi[i] = tr_off(IC<RCA>{}, wave_m + i * 32, tr_row + 4); }
#pragma unroll
    for (int j = 0; j < NI; ++j) { offb_lo[j] = tr_off(IC<RCB>{}, wave_n + j * 32, tr_row); offb_hi[j] = tr_off(IC<RCB>{}, wave_n + j * 32, tr_row + 4); }

    struct Frags { bf16x8 a[MI], b[NI]; };
    // the swizzle depends on row % 4 only and a k-step advances the row by 16: offsets just shift
    auto read_task = [&](auto t, Frags &f, const bf16_t *src_a, const bf16_t *src_b, int ks) __attribute__((always_inline)) {
        constexpr int Tk = decltype(t)::value;
        if constexpr (Tk < MI) {
            const bf16_t *q = src_a + ks * 16 * BMT;
            const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(q + offa_lo[Tk]));
            const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(q + offa_hi[Tk]));
            f.a[Tk] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        } else {
            const bf16_t *q = src_b + ks * 16 * BNT;
            const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(q + offb_lo[Tk - MI]));
            const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(q + offb_hi[Tk - MI]));
            f.b[Tk - MI] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };
    constexpr int N_READ = MI + NI;

    auto mfma_with = [&](const Frags &f, auto ntask, auto &&task) __attribute__((always_inline)) {
        constexpr int NTASK = decltype(ntask)::value;
        static_for<NMF>([&](auto s) __attribute__((always_inline)) {
            constexpr int S = decltype(s)::value;
            acc[S / NI][S % NI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[S / NI], f.b[S % NI], acc[S / NI][S % NI], 0, 0, 0);
            static_for<NTASK>([&](auto t) __attribute__((always_inline)) {
                constexpr int Tk = decltype(t)::value;
                if constexpr (Tk * NMF / NTASK == S) task(t);
            });
            pin();
        });
    };

    // ---- pipeline (same shape as the forward kernel's) --------------------------------------------
    Frags f0, f1;
    static_for<NS>([&](auto s) __attribute__((always_inline)) {
        static_for<L>([&](auto t) __attribute__((always_inline)) { addr_task(t); });
        static_for<L>([&](auto t) __attribute__((always_inline)) { load_task(t, stage_a(s), stage_b(s)); });
    });
    wait_vmcnt<L * (NS - 1)>();
    ring_barrier();
    static_for<N_READ>([&](auto t) __attribute__((always_inline)) { read_task(t, f0, sa0, sb0, 0); });

    auto run_stage = [&](auto s) __attribute__((always_inline)) {
        constexpr int S = decltype(s)::value;
        constexpr int S1 = (S + 1) % NS;
        bf16_t *ca = stage_a(s), *cb = stage_b(s);
        static_for<KS - 1>([&](auto k) __attribute__((always_inline)) {
            constexpr int ks = decltype(k)::value;
            Frags &cur = (ks & 1) ? f1 : f0;
            Frags &nxt = (ks & 1) ? f0 : f1;
            // this k-step's share of the address tasks, spread evenly over k-steps 0..KS-2
            constexpr int a0 = ks * L / (KS - 1), a1 = (ks + 1) * L / (KS - 1);
            mfma_with(cur, IC<N_READ + (a1 - a0)>{}, [&](auto t) __attribute__((always_inline)) {
                constexpr int Tk = decltype(t)::value;
                if constexpr (Tk < N_READ) read_task(t, nxt, ca, cb, ks + 1); else addr_task(IC<a0 + Tk - N_READ>{});
            });
        });
        wait_lgkmcnt0();
        wait_vmcnt<L * (NS - 2)>();
        ring_barrier();
        mfma_with(f1, IC<L + N_READ>{}, [&](auto t) __attribute__((always_inline)) {
            constexpr int Tk = decltype(t)::value;
            if constexpr (Tk < L) load_task(t, ca, cb);
            else read_task(IC<Tk - L>{}, f0, stage_a(IC<S1>{}), stage_b(IC<S1>{}), 0);
        });
    };
    // whole turns of the ring in a loop whose body is one basic block, then the remaining stages
    int kt = 0;
    for (; kt + NS <= KT; kt += NS) static_for<NS>([&](auto s) __attribute__((always_inline)) { run_stage(s); });
    const int rem = KT - kt;
    if (rem >= 1) run_stage(IC<0>{});
    if constexpr (NS > 2) if (rem >= 2) run_stage(IC<1>{});
    if constexpr (NS > 3) if (rem >= 3) run_stage(IC<2>{});
    wait_vmcnt<0>();

    // ---- fp32 partial tile -> workspace ------------------------------------------------------
    // Through LDS, one 32-row block of the wave tile at a time, so that a row's WN columns leave as
    // 16-byte stores (the column count is a multiple of 8, so a group of four is valid or not as one).
    {
        constexpr int RS = 32 * WN * 2;               // staging per wave, in bf16 slots (fp32 = 2 slots)
        constexpr bool USE_A = SZA >= SZB;
        constexpr int SZ = USE_A ? SZA : SZB;
        constexpr int WPB = SZ / RS;
        static_assert(WPB >= 1 && NW <= WPB * NS, "partial-tile staging must fit the stage buffers of one operand");
        constexpr int CPR = WN / 4;                   // float4 groups per staged row
        wait_lgkmcnt0();
        __syncthreads();
        const int bi = wave / WPB;
        bf16_t *sb = bi == 0 ? (USE_A ? sa0 : sb0) : bi == 1 ? (USE_A ? sa1 : sb1) : bi == 2 ? (USE_A ? sa2 : sb2) : (USE_A ? sa3 : sb3);
        float *stg = reinterpret_cast<float *>(sb + (wave % WPB) * RS);
        float *out = p.partial + (size_t)z * p.K * RSC;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
#pragma unroll
            for (int e = 0; e < 16; ++e)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    stg[(8 * (e >> 2) + 4 * (lane >> 5) + (e & 3)) * WN + j * 32 + (lane & 31)] = acc[i][j][e];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int q = 0; q < 32 * CPR / 64; ++q) {
                const int idx = q * 64 + lane;
                const int r = idx / CPR, c4 = idx % CPR;
                const int k = k0 + wave_m + i * 32 + r, c = n0 + wave_n + c4 * 4;
                const float4 v = *reinterpret_cast<const float4 *>(stg + r * WN + c4 * 4);
                if (k < p.K && c < RSC) *reinterpret_cast<float4 *>(out + (size_t)k * RSC + c) = v;
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

// ---- split reduction: dw = sum over splits of the fp32 partial tensors -----------------------------------
// A wave is divided into G groups of 64/G lanes.  The lanes of a group own consecutive outputs (so a group's
// load of one split is one contiguous run); group g adds the splits g, g+G, g+2G, ... in ascending order, and
// the G group sums are then added across the wave with a butterfly of lane exchanges (__shfl_xor over
// 64/G, ..., 32 lanes: DPP / permute instructions, no memory).  The order of additions depends only on G and
// the split count, so results are bit-identical from run to run.  G = 4 for ordinary split counts, 16 when
// many splits meet a small dw (more loads in flight per output).
__device__ __forceinline__ float4 shfl_xor4(const float4 v, int lanes)
{
    return make_float4(__shfl_xor(v.x, lanes), __shfl_xor(v.y, lanes), __shfl_xor(v.z, lanes), __shfl_xor(v.w, lanes));
}

// Plain NHWC operands (source index == destination index), four outputs per lane with 16-byte loads.
// OUT = float: dw in fp32; OUT = bf16_t: the fp32 sum rounded once (nearest even) to bf16
__device__ __forceinline__ void store4(float *dw, int i4, const float4 v) { reinterpret_cast<float4 *>(dw)[i4] = v; }
__device__ __forceinline__ void store4(bf16_t *dw, int i4, const float4 v)
{
    reinterpret_cast<uint2 *>(dw)[i4] = make_uint2((uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16),
                                                   (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16));
}

template <int G, typename OUT>
__global__ __launch_bounds__(256) void wgrad_reduce_vec4_kernel(const float4 *partial, OUT *dw,
                                                                int total4, int splits)
{
    constexpr int LPG = 64 / G;                       // lanes per group
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPG;
    const int gid = (blockIdx.x * 4 + wave) * LPG + lane % LPG;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (gid < total4)
        for (int zz = grp; zz < splits; zz += G) {
            const float4 v = partial[(size_t)zz * total4 + gid];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
#pragma unroll
    for (int d = LPG; d < 64; d <<= 1) {
        const float4 o = shfl_xor4(acc, d);
        acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
    }
    if (grp == 0 && gid < total4) store4(dw, gid, acc);
}

// General form: dw[k][r][s][c] is read back from column (r/d)*col_r + (s/d)*col_s + ((r%d)*d + s%d)*Cq + c of
// partial[z][k][.], d = s2d (1 for everything but space-to-depth operands, where it is the stride).  The
// re-packed operands of odd channel counts have wider columns that are dropped here.  One output per lane.
template <int G, typename OUT>
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float *__restrict__ partial, OUT *__restrict__ dw,
                                                           int total, int splits, int ncols, int RSC, int SC, int C,
                                                           int col_r, int col_s, int s2d, int Cq, size_t split_stride)
{
    constexpr int LPG = 64 / G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPG;
    const int gid = (blockIdx.x * 4 + wave) * LPG + lane % LPG;
    float acc = 0.f;
    if (gid < total) {
        const int k = gid / RSC, rem = gid % RSC;
        const int r = rem / SC, rem2 = rem % SC;
        const int sidx = rem2 / C, c = rem2 % C;
        const size_t src = (size_t)k * ncols + (r / s2d) * col_r + (sidx / s2d) * col_s + ((r % s2d) * s2d + sidx % s2d) * Cq + c;
        for (int zz = grp; zz < splits; zz += G) acc += partial[(size_t)zz * split_stride + src];
    }
#pragma unroll
    for (int d = LPG; d < 64; d <<= 1) acc += __shfl_xor(acc, d);
    if (grp == 0 && gid < total) store_f32(dw + gid, acc);
}

// slots: workgroups that fit one CU; util: fraction of the CU's matrix peak the tile sustains (measured)
struct WgradTile { int bm, bn, bp, slots; float util; const char *name; };
const WgradTile kTiles[] = {
    {128, 128, 64, 2, 0.36f, "wgrad_128x128_p64s2_w4"},
    {256, 256, 32, 1, 0.47f, "wgrad_256x256_p32s4_w8"},
    {256, 128, 32, 1, 0.30f, "wgrad_256x128_p32s4_w8"},
    {128, 256, 32, 1, 0.30f, "wgrad_128x256_p32s4_w8"},
    {64, 64, 64, 4, 0.12f, "wgrad_64x64_p64s2_w4"},
    {64, 128, 64, 2, 0.22f, "wgrad_64x128_p64s2_w4"},
    {128, 64, 64, 2, 0.22f, "wgrad_128x64_p64s2_w4"},
    {256, 256, 64, 1, 0.01f, "wgrad_256x256_p64s2_w8"},
    {128, 128, 32, 2, 0.01f, "wgrad_128x128_p32s4_w4"},
};
constexpr int N_TILES = sizeof(kTiles) / sizeof(kTiles[0]);

template <int BMT, int BNT, int BP, int NS, int WR, int WC>
int launch(const WgradParams &p, int tiles, hipStream_t st)
{
    WgradParams q = p;
    q.tiles = tiles;
    q.n_wg = tiles * p.splits;
    const int grid = (q.n_wg + 7) / 8 * 8;
    hipLaunchKernelGGL((wgrad_kernel<BMT, BNT, BP, NS, WR, WC>), dim3((unsigned)grid), dim3(64 * WR * WC), 0, st, q);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

int launch_choice(int idx, const WgradParams &p, int tiles, hipStream_t st)
{
    switch (idx) {
    case 0: return launch<128, 128, 64, 2, 2, 2>(p, tiles, st);
    case 1: return launch<256, 256, 32, 4, 2, 4>(p, tiles, st);
    case 2: return launch<256, 128, 32, 4, 4, 2>(p, tiles, st);
    case 3: return launch<128, 256, 32, 4, 2, 4>(p, tiles, st);
    case 4: return launch<64, 64, 64, 2, 2, 2>(p, tiles, st);
    case 5: return launch<64, 128, 64, 2, 2, 2>(p, tiles, st);
    case 6: return launch<128, 64, 64, 2, 2, 2>(p, tiles, st);
    case 7: return launch<256, 256, 64, 2, 2, 4>(p, tiles, st);
    default: return launch<128, 128, 32, 4, 2, 2>(p, tiles, st);
    }
}

struct Plan { int tile, k_tiles, n_tiles, splits, span; };

// Tile and split choice: the pair with the least modelled time - rounds over the chip's workgroup
// slots (256 CUs x slots per CU) x stages each split walks x time per stage, plus the traffic of
// writing and re-reading one fp32 partial tensor per split.  MXC_FORCE_WGRAD=<name> (tuning sweeps
// only) fixes the tile.
Plan search_plan(const WgradGeom &g, int forced, int forced_splits);

#include "tuned_wgrad.inc"

int tile_index(const char *name, size_t len)
{
    for (int i = 0; i < N_TILES; ++i)
        if (strlen(kTiles[i].name) == len && !strncmp(name, kTiles[i].name, len)) return i;
    return -1;
}

// Tile and split count, in this order: MXC_FORCE_WGRAD=<tile>[/<splits>] (tuning sweeps only); the table of
// measured best choices (tuned_wgrad.inc, written by the tuning script from timings on the device) when it
// holds this geometry; else the time model's search.  The search costs tens of microseconds, a call needs
// its answer up to three times (size query, workspace carve-out, launch) and a training loop asks for the
// same few geometries over and over: the calling thread keeps its answers (no locks; 32 entries,
// overwritten in turn).
Plan make_plan(const WgradGeom &g)
{
    int forced = -1, forced_splits = 0;
    if (const char *f = getenv("MXC_FORCE_WGRAD")) {
        const char *slash = strchr(f, '/');
        forced = tile_index(f, slash ? (size_t)(slash - f) : strlen(f));
        if (forced >= 0 && slash) forced_splits = atoi(slash + 1);
    } else {
        for (const TunedWgrad &e : kTunedWgrad)
            if (e.N == g.N && e.H == g.oH && e.W == g.oW && e.C == g.C && e.K == g.K && e.R == g.R && e.S == g.S &&
                e.stride == g.ostride && e.pad == g.opad) {
                forced = tile_index(e.tile, strlen(e.tile));
                forced_splits = forced >= 0 ? e.splits : 0;
                break;
            }
    }
    struct Entry { WgradGeom g; int forced, forced_splits; Plan plan; bool used; };
    static thread_local Entry cache[32] = {};
    static thread_local int next = 0;
    for (const Entry &e : cache)
        if (e.used && e.forced == forced && e.forced_splits == forced_splits && !memcmp(&e.g, &g, sizeof(WgradGeom))) return e.plan;
    Entry &slot = cache[next];
    next = (next + 1) % 32;
    slot.g = g; slot.forced = forced; slot.forced_splits = forced_splits; slot.plan = search_plan(g, forced, forced_splits);
    slot.used = true;
    return slot.plan;
}

Plan search_plan(const WgradGeom &g, int forced, int forced_splits)
{
    const int RSC = g.TR * g.TS * g.run;
    const long long M = (long long)g.N * g.P * g.Q;
    Plan best_pl{};
    double best = 1e300;
    for (int t = 0; t < N_TILES; ++t) {
        if (forced >= 0 && t != forced) continue;
        const WgradTile &tc = kTiles[t];
        // no tile dimension (beyond 64) more than a third larger than the problem's: past that the padding
        // rows cost more than the larger tile gains
        if (forced < 0 && ((tc.bm > 64 && tc.bm * 3 > g.K * 4) || (tc.bn > 64 && tc.bn * 3 > RSC * 4))) continue;
        const int k_tiles = (g.K + tc.bm - 1) / tc.bm, n_tiles = (RSC + tc.bn - 1) / tc.bn;
        const long long tiles = (long long)k_tiles * n_tiles;
        const long long slots = 256LL * tc.slots;
        const double stage_us = 2.0 * tc.bm * tc.bn * tc.bp * tc.slots / (2.5e15 / 256 * tc.util) * 1e6;
        const double split_us = (double)g.K * RSC * 8.0 / 3e12 * 1e6;
        long long max_splits = (M + 2LL * tc.bp - 1) / (2LL * tc.bp);
        if (max_splits > 1024) max_splits = 1024;
        if (max_splits < 1) max_splits = 1;
        for (long long sp = 1; sp <= max_splits; ++sp) {
            if (forced_splits > 0 && sp != (forced_splits < max_splits ? forced_splits : max_splits)) continue;
            const long long wgs = tiles * sp, rounds = (wgs + slots - 1) / slots;
            const long long stages = ((M + sp - 1) / sp + tc.bp - 1) / tc.bp;
            const double t_us = (double)rounds * (double)(stages + 6) * stage_us + (double)sp * split_us;
            if (t_us < best) {
                best = t_us;
                long long span = (M + sp - 1) / sp;
                span = (span + tc.bp - 1) / tc.bp * tc.bp;
                best_pl = Plan{t, k_tiles, n_tiles, (int)((M + span - 1) / span), (int)span};
            }
        }
    }
    return best_pl;
}

}  // namespace

const char *wgrad_tile_name(int index) { return index >= 0 && index < N_TILES ? kTiles[index].name : nullptr; }

WgradGeom wgrad_geom_plain(const ConvShape &s)
{
    return WgradGeom{s.N, s.H, s.W, s.C, s.K, s.P, s.Q, s.stride, s.pad, s.R, s.S, s.C, s.R, s.S, s.C, s.S * s.C, s.C, 1, 0, s.H, s.W, s.stride, s.pad};
}

WgradGeom wgrad_geom_chanpad(const ConvShape &s)
{
    const int C8 = (s.C + 7) / 8 * 8;
    return WgradGeom{s.N, s.H, s.W, C8, s.K, s.P, s.Q, s.stride, s.pad, s.R, s.S, C8, s.R, s.S, s.C, s.S * C8, C8, 1, 0, s.H, s.W, s.stride, s.pad};
}

WgradGeom wgrad_geom_smallc(const ConvShape &s)
{
    const SmallCGeom g = smallc_geom(s);
    return WgradGeom{s.N, g.Hp, g.Wp, g.pix, s.K, s.P, s.Q, s.stride, 0, s.R, 1, g.run, s.R, s.S, s.C, g.run, g.pix, 1, 0, s.H, s.W, s.stride, s.pad};
}

WgradGeom wgrad_geom_s2d(const ConvShape &s)
{
    const S2DGeom g = s2d_geom(s);
    return WgradGeom{s.N, g.H2, g.W2, g.C2, s.K, s.P, s.Q, 1, 0, g.R2, g.S2, g.C2, s.R, s.S, s.C, g.S2 * g.C2, g.C2, g.s, g.Cq, s.H, s.W, s.stride, s.pad};
}

bool wgrad_supported(const WgradGeom &g)
{
    const long long M = (long long)g.N * g.P * g.Q;
    return g.pix % 4 == 0 && g.run % 8 == 0 && g.K % 8 == 0 && M < 0x7FFF0000ll &&
           (long long)g.N * g.H * g.W * g.pix * 2 < 0x7FFF0000ll && M * g.K * 2 < 0x7FFF0000ll && g.H + g.TR + g.pad <= 8192 &&
           g.W + g.TS + g.pad <= 8192 && (long long)g.P * g.stride <= 8192 && (long long)g.Q * g.stride <= 8192 &&
           (long long)g.K * g.TR * g.TS * g.run < 0x7FFFFFFFll;
}

size_t wgrad_workspace(const WgradGeom &g)
{
    return (size_t)make_plan(g).splits * g.K * g.TR * g.TS * g.run * sizeof(float);
}

template <typename OUT>
static int launch_reduce(const WgradGeom &g, float *partial, OUT *dw, int splits, int ncols, bool identity, hipStream_t st)
{
    const int total = g.K * g.R * g.S * g.C;
    // many splits of a small dw: 16 lane groups keep enough loads in flight; otherwise 4
    const bool wide = splits >= 32 && total < 256 * 1024;
    if (!identity && splits > 1) {
        // Packed geometries (first layers): the column remap reads single floats, so first add the splits with the
        // 16-byte kernel - in place, into the first split's partial tensor: every element is read and then written
        // by the same lane group - and remap that one tensor afterwards.
        const int cols4 = g.K * ncols / 4;            // ncols is a multiple of 8
        if (wide)
            hipLaunchKernelGGL((wgrad_reduce_vec4_kernel<16, float>), dim3((unsigned)((cols4 + 15) / 16)), dim3(256), 0, st,
                               (const float4 *)partial, partial, cols4, splits);
        else
            hipLaunchKernelGGL((wgrad_reduce_vec4_kernel<4, float>), dim3((unsigned)((cols4 + 63) / 64)), dim3(256), 0, st,
                               (const float4 *)partial, partial, cols4, splits);
        if (hipGetLastError() != hipSuccess) return MXC_ERR_LAUNCH;
        splits = 1;
    }
    if (identity && total % 4 == 0) {
        const int total4 = total / 4;
        if (wide)
            hipLaunchKernelGGL((wgrad_reduce_vec4_kernel<16, OUT>), dim3((unsigned)((total4 + 15) / 16)), dim3(256), 0, st,
                               (const float4 *)partial, dw, total4, splits);
        else
            hipLaunchKernelGGL((wgrad_reduce_vec4_kernel<4, OUT>), dim3((unsigned)((total4 + 63) / 64)), dim3(256), 0, st,
                               (const float4 *)partial, dw, total4, splits);
    } else if (wide) {
        hipLaunchKernelGGL((wgrad_reduce_kernel<16, OUT>), dim3((unsigned)((total + 15) / 16)), dim3(256), 0, st, partial, dw, total,
                           splits, ncols, g.R * g.S * g.C, g.S * g.C, g.C, g.col_r, g.col_s, g.s2d, g.Cq, (size_t)g.K * ncols);
    } else {
        hipLaunchKernelGGL((wgrad_reduce_kernel<4, OUT>), dim3((unsigned)((total + 63) / 64)), dim3(256), 0, st, partial, dw, total,
                           splits, ncols, g.R * g.S * g.C, g.S * g.C, g.C, g.col_r, g.col_s, g.s2d, g.Cq, (size_t)g.K * ncols);
    }
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

int wgrad(const WgradGeom &g, const void *x, const void *dy, void *dw, bool dw_bf16, float *partial, hipStream_t st,
          const char **variant)
{
    const Plan pl = make_plan(g);
    const WgradTile &tc = kTiles[pl.tile];
    WgradParams p{};
    p.x = (const bf16_t *)x; p.dy = (const bf16_t *)dy; p.partial = partial;
    p.N = g.N; p.H = g.H; p.W = g.W; p.pix = g.pix; p.K = g.K; p.P = g.P; p.Q = g.Q;
    p.stride = g.stride; p.pad = g.pad;
    p.TS = g.TS; p.run = g.run; p.ncols = g.TR * g.TS * g.run;
    p.n_tiles = pl.n_tiles;
    p.splits = pl.splits;
    p.span = pl.span;
    p.M = g.N * g.P * g.Q;
    p.dq = tc.bp % g.Q;
    const int rows = tc.bp / g.Q;
    p.dp = rows % g.P;
    p.dn = rows / g.P;
    p.x_bytes = (unsigned)((long long)g.N * g.H * g.W * g.pix * 2);
    p.dy_bytes = (unsigned)((long long)p.M * g.K * 2);
    const long long tiles = (long long)pl.k_tiles * pl.n_tiles;
    if (tiles * p.splits > 0x3FFFFFFFll) return MXC_ERR_SHAPE;
    const bool identity = g.s2d == 1 && g.col_s == g.C && g.col_r == g.S * g.C && p.ncols == g.R * g.S * g.C;
    // one split whose columns are already in KRSC order and an fp32 result: the "partial" tensor is dw itself
    const bool direct = p.splits == 1 && identity && !dw_bf16;
    if (direct) p.partial = (float *)dw;
    const int rc = launch_choice(pl.tile, p, (int)tiles, st);
    if (rc != MXC_OK) return rc;
    *variant = tc.name;
    if (direct) return MXC_OK;
    return dw_bf16 ? launch_reduce(g, p.partial, (bf16_t *)dw, p.splits, p.ncols, identity, st)
                   : launch_reduce(g, p.partial, (float *)dw, p.splits, p.ncols, identity, st);
}

}  // namespace mxc
