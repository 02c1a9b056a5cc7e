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
// Tiling: a workgroup of 4 or 8 waves owns a BM x BN output tile; each wave accumulates a
// (BM/WR) x (BN/WC) sub-tile with v_mfma_f32_32x32x16_bf16 in fp32.  The reduction advances in
// steps of BKT (32 or 64) through a ring of NS LDS stages that are filled by direct global->LDS
// loads issued NS stages ahead of their use; 16-byte chunks are XOR-swizzled by row so that the
// ds_read_b128 operand fetches are bank-conflict free.
//
// Reduction order: tap-major as the filter matrix is laid out, or, when Ci is a multiple of the
// step, channel-block-major (all taps of a 64-channel block back to back: better L2 reuse).
// Problems with few tiles and a long reduction (FullyConnected shapes) split the reduction over
// workgroups into fp32 partial tiles that a finishing kernel adds in a fixed order.  A large 1x1
// filter can be read in place for backward-data (BT kernels: transposed LDS tiles).  The epilogue
// can add a bias, apply ReLU, and zero results under a mask.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <type_traits>

#include "mxc_internal.h"

namespace mxc {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16x4 __attribute__((address_space(3))) * lds_bf16x4_ptr;

typedef __attribute__((address_space(3))) void *lds_vptr;
typedef short s16x2 __attribute__((ext_vector_type(2)));

constexpr unsigned OOB = 0x80000000u;   // a buffer offset no operand reaches: the load returns zeros


template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ void wait_lgkmcnt0() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void pin() { __builtin_amdgcn_sched_barrier(0); }   // nothing is scheduled across
// Workgroup barrier of the ring: the bare instruction, with the counters it needs waited for by hand just before
// it.  __syncthreads() would add a release fence, which the compiler turns into a wait for every outstanding
// global->LDS load (vmcnt(0)) - that empties a ring of more than two stages at every stage.
__device__ __forceinline__ void ring_barrier() { pin(); __builtin_amdgcn_s_barrier(); pin(); }

template <int I> using IC = std::integral_constant<int, I>;

// Transposed filter tiles (BT kernels): XOR applied to the chunk index of tile row `row` (RC chunks of
// 16 bytes per row) so that the four rows touched by one transposing read fall into different banks.
template <int RC> __device__ __forceinline__ int bt_row_swz(int row)
{
    if constexpr (RC >= 16) return (row & 3) << 2;
    else if constexpr (RC == 8) return ((row >> 1) & 1) << 2;
    else return 0;
}
template <class F, int... I> __device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) { (f(IC<I>{}), ...); }
template <int N, class F> __device__ __forceinline__ void static_for(F &&f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }

// BM x BN output tile, BKT reduction elements per stage, NS stages, WR x WC waves.  The register
// budget is set for two waves per SIMD when the workgroup has 4 waves and its LDS lets two of them
// share a CU.
// BT = true: the filter operand is read transposed, straight from w[K][Co] (1x1 filters): its LDS tile is
// [reduction row][BN output columns] and its MFMA fragments come from ds_read_b64_tr_b16.
// TI = true: channel-block-major reduction order (needs Ci % BKT == 0); a compile-time choice so that the
// stage body is one basic block and the pinned interleave of address work and MFMAs survives.
template <int BM, int BN, int BKT, int NS, int WR, int WC, bool BT, bool TI>
__global__ __launch_bounds__(64 * WR * WC, (WR * WC == 4 && NS * (BM + BN) * BKT * 2 <= 80 * 1024) ? 2 : 1) void igemm_kernel(
    const IgemmParams p)
{
    static_assert(!(BT && TI), "the in-place filter variant has one tap");
    constexpr int NW = WR * WC, NT = 64 * NW;
    constexpr int WM = BM / WR, WN = BN / WC;     // wave tile
    constexpr int MI = WM / 32, NI = WN / 32;     // 32x32 MFMA blocks per wave
    constexpr int NMF = MI * NI;                  // MFMAs per k-step
    constexpr int CH = BKT / 8;                   // 16-byte chunks per tile row
    constexpr int RPL = 64 / CH;                  // tile rows filled by one wave-wide load
    constexpr int RB = 256 / (BKT * 2);           // tile rows per 256-byte span of LDS banks
    constexpr int A_LD = BM / RPL / NW;           // wave-wide loads per wave per stage
    constexpr int B_LD = BN / RPL / NW;
    constexpr int L = A_LD + B_LD;
    constexpr int KS = BKT / 16;                  // MFMA k-steps per stage
    static_assert(BKT == 32 || BKT == 64, "BKT");
    static_assert(NS >= 2 && NS <= 4, "NS");
    static_assert(NW % 2 == 0 && BM % (RPL * NW) == 0 && BN % (RPL * NW) == 0, "tile/wave mismatch");
    static_assert(L * (NS - 1) < 64, "vmcnt range");
    static_assert(KS % 2 == 0, "fragment ping-pong assumes an even number of k-steps");
    constexpr int RCB = BN / 8;                   // BT: 16-byte chunks per filter-tile row
    constexpr int RPLB = 64 / RCB;                // BT: filter-tile rows filled by one wave-wide load
    static_assert(!BT || (BKT == 64 && RCB >= 4 && RCB <= 32 && BKT % (RPLB * NW) == 0 && BKT / RPLB / NW == B_LD), "BT tile/wave mismatch");

    // Every stage is its own LDS object (not one array indexed by the stage): the compiler can then
    // see that the direct loads filling one stage never alias the operand reads of another and does
    // not serialise them.
    constexpr int SZA = BM * BKT, SZB = BN * BKT;
    __shared__ __attribute__((aligned(1024))) bf16_t sa0[SZA];
    __shared__ __attribute__((aligned(1024))) bf16_t sa1[SZA];
    __shared__ __attribute__((aligned(1024))) bf16_t sa2[NS > 2 ? SZA : 8];
    __shared__ __attribute__((aligned(1024))) bf16_t sa3[NS > 3 ? SZA : 8];
    __shared__ __attribute__((aligned(1024))) bf16_t sb0[SZB];
    __shared__ __attribute__((aligned(1024))) bf16_t sb1[SZB];
    __shared__ __attribute__((aligned(1024))) bf16_t sb2[NS > 2 ? SZB : 8];
    __shared__ __attribute__((aligned(1024))) bf16_t sb3[NS > 3 ? SZB : 8];
    // per tap: .x = byte offset of the tap relative to tap 0, .y = (dh, dv) packed as two int16
    __shared__ int2 tap_tab[MAX_TAPS + 1];
    auto stage_a = [&](auto s) __attribute__((always_inline)) -> bf16_t * {
        constexpr int S = decltype(s)::value;
        if constexpr (S == 0) return sa0; else if constexpr (S == 1) return sa1; else if constexpr (S == 2) return sa2; else return sa3;
    };
    auto stage_b = [&](auto s) __attribute__((always_inline)) -> bf16_t * {
        constexpr int S = decltype(s)::value;
        if constexpr (S == 0) return sb0; else if constexpr (S == 1) return sb1; else if constexpr (S == 2) return sb2; else return sb3;
    };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps LDS targets in SGPRs
    const int wave_m = (wave / WC) * WM, wave_n = (wave % WC) * WN;

    // Workgroup -> tile.  Consecutive workgroup ids are dealt round-robin to the 8 XCDs; give each
    // XCD a contiguous range of tiles, n-tile fastest, so that tiles sharing an activation tile meet
    // in one L2.
    const int total = p.m_tiles * p.n_tiles;
    const int units = total * (p.splits > 1 ? p.splits : 1);
    const int per_xcd = (units + 7) / 8;
    const int unit = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (unit >= units) return;
    const int logical = unit % total, split_z = unit / total;
    const int m0 = p.m_begin + (logical / p.n_tiles) * BM, n0 = (logical % p.n_tiles) * BN;

    const int T = p.TR * p.TS;
    const int Kd = T * p.Ci;
    const int KT = (Kd + BKT - 1) / BKT;

    // ---- tap table -------------------------------------------------------------------------------
    // Entry T is a sentinel whose row offset lies far outside any image: every chunk past the end
    // of the reduction fails the bounds test and is filled with zeros.
    for (int t = tid; t <= T; t += NT) {
        int2 e;
        if (t < T) {
            const int dh = (p.tap_row_inner ? t % p.TR : t / p.TS) * p.tstep_h;
            const int dv = (p.tap_row_inner ? t / p.TR : t % p.TS) * p.tstep_w;
            e.x = ((dh * p.Wi + dv) * p.pix) * 2;
            e.y = (dh & 0xFFFF) | (dv << 16);
        } else {
            e.x = 0;
            e.y = (-16384) & 0xFFFF;
        }
        tap_tab[t] = e;
    }

    // ---- load bookkeeping --------------------------------------------------------------------
    // Wave-wide load number i fills tile rows RPL*i .. RPL*i+RPL-1: lane l -> row RPL*i + l/CH, chunk
    // position l%CH.  Chunk c of row r lives at position c ^ ((r/RB) % CH), which spreads any 16
    // consecutive rows of one logical chunk over all 64 banks.  This wave issues loads wave, wave+NW,
    // ...; (RPL/RB)*NW is a multiple of CH, so the logical chunk (= reduction offset) a lane fetches is
    // the same for all of them.
    const int ld_sub = lane / CH;
    const int ld_chunk = (lane % CH) ^ (((RPL / RB) * wave + ld_sub / RB) % CH);

    const buf_rsrc_t rs_in = make_buf_rsrc(p.in, p.in_bytes);
    const buf_rsrc_t rs_wm = make_buf_rsrc(p.wm, p.wm_bytes);

    int a_off[A_LD];     // byte offset of (n, base_h, base_w, 0) in `in` (may be negative)
    int a_hw[A_LD];      // base_h (low 16 bits) and base_w (high 16), signed; invalid row: h = -16384
#pragma unroll
    for (int i = 0; i < A_LD; ++i) {
        const int m = m0 + RPL * (wave + NW * i) + ld_sub;
        if (m < p.m_end) {
            const unsigned b = (unsigned)m % (unsigned)p.Mw, t2 = (unsigned)m / (unsigned)p.Mw;
            const unsigned a = t2 % (unsigned)p.Mh, n = t2 / (unsigned)p.Mh;
            const int h = (int)a * p.in_mul_h + p.in_off_h, w = (int)b * p.in_mul_w + p.in_off_w;
            a_off[i] = (int)((((long long)n * p.Hi + h) * p.Wi + w) * p.pix * 2);
            a_hw[i] = (h & 0xFFFF) | (w << 16);
        } else {
            a_off[i] = 0;
            a_hw[i] = (-16384) & 0xFFFF;
        }
    }
    unsigned b_off[B_LD];   // byte offset of the filter row, OOB for rows past Co
    // BT: lane -> row RPLB*i' + lane/RCB of the stage's 64 reduction rows, output-column chunk lane%RCB (swizzled);
    // b_off = byte offset of (row, column chunk) relative to the stage's first filter row
    [[maybe_unused]] const int lb_sub = lane / RCB;
    [[maybe_unused]] const int lb_chunk = (lane % RCB) ^ bt_row_swz<RCB>(RPLB * wave + lb_sub);   // RPLB*NW*i never changes the swizzle
    [[maybe_unused]] const bool bt_col_ok = n0 + lb_chunk * 8 < p.Co;
#pragma unroll
    for (int i = 0; i < B_LD; ++i) {
        if constexpr (BT) {
            b_off[i] = (unsigned)((RPLB * (wave + NW * i) + lb_sub) * p.Co * 2 + (n0 + lb_chunk * 8) * 2);
        } else {
            const int co = n0 + RPL * (wave + NW * i) + ld_sub;
            b_off[i] = co < p.Co ? (unsigned)co * (unsigned)Kd * 2u : OOB;
        }
    }
    // Reduction position of this lane's chunk: kd = stage*BKT + ld_chunk*8 = tap*Ci + ci, kept as
    // (tap, ci) and advanced without branches: BKT = kq*Ci + kr.
    const int kq = BKT / p.Ci, kr2 = (BKT % p.Ci) * 2, Ci2 = p.Ci * 2, Kd2 = Kd * 2;
    // first stage and number of stages of this workgroup (all of them unless the reduction is split)
    const int k_lo = p.splits > 1 ? split_z * p.split_stages : 0;
    const int k_cnt = p.splits > 1 ? min(KT - k_lo, p.split_stages) : KT;
    const int kd0 = k_lo * BKT + ld_chunk * 8;     // this lane's reduction position in the first stage (tap-major order)
    int kd2 = kd0 * 2;                             // byte offset within a filter row
    int ci2 = (kd0 % p.Ci) * 2, tap = kd0 / p.Ci;
    if constexpr (TI) {                            // stage s = (channel block s / T, tap s % T)
        tap = k_lo % T;
        ci2 = (k_lo / T) * (BKT * 2) + ld_chunk * 16;
    }
    const int lim_hw = ((p.Hi - 1) & 0xFFFF) | ((p.Wi - 1) << 16);

    unsigned va[A_LD], vb[B_LD];   // byte offsets of the next stage's loads

    // address generation for the next stage, split in A_LD + 1 small tasks so that it can be spread
    // between MFMAs.  tap_e is the tap-table entry of the stage the addresses are for; the last task
    // advances the reduction position and fetches the entry of the stage after, a whole stage before
    // the first task that reads it.
    int2 tap_e = make_int2(0, 0);
    auto fetch_tap = [&]() __attribute__((always_inline)) { tap_e = tap_tab[tap < T ? tap : T]; };
    auto addr_task = [&](auto t) __attribute__((always_inline)) {
        constexpr int Tk = decltype(t)::value;
        if constexpr (Tk < A_LD) {
            constexpr int i = Tk;
            const s16x2 hw = __builtin_bit_cast(s16x2, a_hw[i]) + __builtin_bit_cast(s16x2, tap_e.y);
            const s16x2 d = __builtin_bit_cast(s16x2, lim_hw) - hw;
            const int bad = (__builtin_bit_cast(int, hw) | __builtin_bit_cast(int, d)) & (int)0x80008000;
            va[i] = bad == 0 ? (unsigned)(a_off[i] + tap_e.x + ci2) : OOB;
        } else {
            if constexpr (BT) {
                // one tap: stage s covers filter rows 64*s .. 64*s+63; kd2 tracks this lane's byte offset 2*(64*s + chunk*8)
                const bool ok = bt_col_ok && kd2 < Kd2;
                const unsigned base = (unsigned)((kd2 - ld_chunk * 16) / 2) * (unsigned)(p.Co * 2);
#pragma unroll
                for (int i = 0; i < B_LD; ++i) vb[i] = ok ? b_off[i] + base : OOB;
                kd2 += BKT * 2;
                ci2 += kr2;
                const int carry = ci2 >= Ci2 ? 1 : 0;
                ci2 -= carry ? Ci2 : 0;
                tap += kq + carry;
            } else if constexpr (TI) {
                // Order (channel block, tap): the pixels a workgroup reads for one channel block serve all
                // its taps back to back, so they are still in the XCD's L2 when the next tap asks for them.
                const bool k_ok = tap < T;
                const unsigned kd = (unsigned)(tap * Ci2 + ci2);
#pragma unroll
                for (int i = 0; i < B_LD; ++i) vb[i] = k_ok ? b_off[i] + kd : OOB;
                const int last = tap + 1 >= T ? 1 : 0;           // wrap to the next channel block
                tap = last ? 0 : tap + 1;
                ci2 += last ? BKT * 2 : 0;
                tap = ci2 >= Ci2 ? T : tap;                       // past the last block: the sentinel tap, for good
            } else {
                const bool k_ok = kd2 < Kd2;
#pragma unroll
                for (int i = 0; i < B_LD; ++i) vb[i] = k_ok ? b_off[i] + (unsigned)kd2 : OOB;
                // advance (tap, ci) and kd by one stage
                kd2 += BKT * 2;
                ci2 += kr2;
                const int carry = ci2 >= Ci2 ? 1 : 0;
                ci2 -= carry ? Ci2 : 0;
                tap += kq + carry;
            }
            fetch_tap();
        }
    };
    constexpr int N_ADDR = A_LD + 1;
    auto load_task = [&](auto t, bf16_t *dst_a, bf16_t *dst_b) __attribute__((always_inline)) {
        constexpr int Tk = decltype(t)::value;
        if constexpr (Tk < A_LD) lds_dma16(rs_in, va[Tk], dst_a + (wave + NW * Tk) * RPL * BKT);
        else lds_dma16(rs_wm, vb[Tk - A_LD], dst_b + (wave + NW * (Tk - A_LD)) * (BT ? RPLB * BN : RPL * BKT));
    };

    // this thread's share of the tile's bias vector (column n0 + tid), requested now, used after the loop
    static_assert(NT >= BN, "one bias value per thread");
    const float bias_t = (p.bias != nullptr && tid < BN && n0 + tid < p.Co) ? p.bias[n0 + tid] : 0.f;

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // operand fetch: lane -> tile row lane%32 of a 32-row block, 8-element group lane/32 of a 16-wide k-step
    const int frag_row = lane & 31, frag_kg = lane >> 5;
    const int frag_swz = (frag_row / RB) % CH;     // block bases are multiples of 32 rows
    const int a_lane = (wave_m + frag_row) * BKT, b_lane = (wave_n + frag_row) * BKT;

    // BT: transposing-read geometry (16-lane group g, lane j16 within it; one read covers 4 reduction rows x
    // 16 output columns): element offsets of the two reads of a 16-row k-step for each of the NI column blocks
    [[maybe_unused]] int bt_lo[NI], bt_hi[NI];
    if constexpr (BT) {
        const int g = lane >> 4, j16 = lane & 15;
        const int tr_row = (g >> 1) * 8 + (j16 >> 2);
        const int tr_ch = (g & 1) * 16 + (j16 & 3) * 4;
        auto tr_off = [&](int ch_base, int row) __attribute__((always_inline)) {
            const int ch = ch_base + tr_ch;
            return row * BN + (((ch >> 3) ^ bt_row_swz<RCB>(row)) << 3) + (ch & 7);
        };
#pragma unroll
        for (int j = 0; j < NI; ++j) { bt_lo[j] = tr_off(wave_n + j * 32, tr_row); bt_hi[j] = tr_off(wave_n + j * 32, tr_row + 4); }
    }
    struct Frags { bf16x8 a[MI], b[NI]; };
    auto read_task = [&](auto t, Frags &f, const bf16_t *src_a, const bf16_t *src_b, int ks) __attribute__((always_inline)) {
        constexpr int Tk = decltype(t)::value;
        const int pos = ((ks * 2 + frag_kg) ^ frag_swz) << 3;
        if constexpr (Tk < MI) f.a[Tk] = *reinterpret_cast<const bf16x8 *>(src_a + a_lane + Tk * 32 * BKT + pos);
        else if constexpr (BT) {
            const bf16_t *q = src_b + ks * 16 * BN;
            const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(q + bt_lo[Tk - MI]));
            const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(q + bt_hi[Tk - MI]));
            f.b[Tk - MI] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        } else f.b[Tk - MI] = *reinterpret_cast<const bf16x8 *>(src_b + b_lane + (Tk - MI) * 32 * BKT + pos);
    };
    constexpr int N_READ = MI + NI;

    // NMF MFMAs of one k-step with `NTASK` side tasks spread between them (program order is pinned:
    // the matrix pipe executes one MFMA while the wave issues the side work behind it)
    // The first NFRONT tasks (operand fetches, which the next k-step waits for) go behind the first half
    // of the MFMAs, the rest behind the second half.
    auto mfma_with = [&](const Frags &f, auto nfront, auto ntask, auto &&task) __attribute__((always_inline)) {
        constexpr int NFRONT = decltype(nfront)::value, NTASK = decltype(ntask)::value;
        constexpr int H1 = NMF > 1 ? NMF / 2 : 1, H2 = NMF - H1 > 0 ? NMF - H1 : 1;
        static_for<NMF>([&](auto s) __attribute__((always_inline)) {
            constexpr int S = decltype(s)::value;
            // filter fragment first: the product is formed transposed, D[co][pixel] (see the epilogue)
            acc[S / NI][S % NI] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[S % NI], f.a[S / NI], acc[S / NI][S % NI], 0, 0, 0);
            static_for<NTASK>([&](auto t) __attribute__((always_inline)) {
                constexpr int Tk = decltype(t)::value;
                constexpr int slot = Tk < NFRONT ? Tk * H1 / NFRONT
                                                 : (NMF > 1 ? H1 + (Tk - NFRONT) * H2 / (NTASK - NFRONT > 0 ? NTASK - NFRONT : 1) : 0);
                if constexpr (slot == S) task(t);
            });
            pin();
        });
    };

    // ---- pipeline ------------------------------------------------------------------------------
    // Stage s lives in ring slot s % NS.  While stage kt is being multiplied, stages kt+1..kt+NS-1
    // are landing.  Per stage: k-steps 0..KS-2 fetch the next k-step's operands, and the one before
    // last also computes the addresses of the refill; then this wave's loads of stage kt+1 are
    // awaited (all but the (NS-2)*L youngest), one barrier publishes stage kt+1 and frees slot
    // kt % NS, and the last k-step's MFMAs run interleaved with the refill loads (stage kt+NS) and the
    // first operand fetch of stage kt+1 - the matrix pipe has work across the barrier.
    Frags f0, f1;
    __syncthreads();   // tap table visible
    fetch_tap();
    static_for<NS>([&](auto s) __attribute__((always_inline)) {
        static_for<N_ADDR>([&](auto t) __attribute__((always_inline)) { addr_task(t); });
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
            constexpr int a0 = ks * N_ADDR / (KS - 1), a1 = (ks + 1) * N_ADDR / (KS - 1);
            mfma_with(cur, IC<N_READ>{}, IC<N_READ + (a1 - a0)>{}, [&](auto t) __attribute__((always_inline)) {
                constexpr int Tk = decltype(t)::value;
                if constexpr (Tk < N_READ) read_task(t, nxt, ca, cb, ks + 1); else addr_task(IC<a0 + Tk - N_READ>{});
            });
        });
        // the last k-step's operands are in f1; all reads of this slot must have returned before it is refilled
        wait_lgkmcnt0();
        wait_vmcnt<L * (NS - 2)>();
        ring_barrier();
        mfma_with(f1, IC<N_READ>{}, IC<N_READ + L>{}, [&](auto t) __attribute__((always_inline)) {
            constexpr int Tk = decltype(t)::value;
            if constexpr (Tk < N_READ) read_task(t, f0, stage_a(IC<S1>{}), stage_b(IC<S1>{}), 0);
            else load_task(IC<Tk - N_READ>{}, ca, cb);
        });
    };

    // Whole turns of the ring in a loop whose body is one basic block (the compiler's own wait insertion for
    // LDS reads against in-flight global->LDS loads merges states at every control-flow join; a join inside
    // the loop makes it wait for all loads at the loop head), then the remaining stages.
    int kt = 0;
    for (; kt + NS <= k_cnt; kt += NS) static_for<NS>([&](auto s) __attribute__((always_inline)) { run_stage(s); });
    const int rem = k_cnt - kt;
    if (rem >= 1) run_stage(IC<0>{});
    if constexpr (NS > 2) if (rem >= 2) run_stage(IC<1>{});
    if constexpr (NS > 3) if (rem >= 3) run_stage(IC<2>{});
    wait_vmcnt<0>();   // drain the zero-fill loads of the stages past the end before the tile's LDS is abandoned

    // ---- epilogue: fp32 -> bf16 (RNE), to the output pixels ------------------------------------
    // The product was formed transposed (filter fragment as the first MFMA operand): accumulator element e of a
    // 32x32 block belongs to tile row lane%32 and column 8*(e/4) + 4*(lane/32) + e%4, so a lane holds runs of four
    // neighbouring output columns of one pixel.
    auto out_pixel = [&](int m) __attribute__((always_inline)) -> long long {
        if (p.linear_out) return m;
        const unsigned b = (unsigned)m % (unsigned)p.Mw, t2 = (unsigned)m / (unsigned)p.Mw;
        const unsigned a = t2 % (unsigned)p.Mh, n = t2 / (unsigned)p.Mh;
        return ((long long)n * p.Ho + ((int)a * p.out_mul_h + p.out_off_h)) * p.Wo + ((int)b * p.out_mul_w + p.out_off_w);
    };
    if (p.splits > 1 || p.f32_out) {
        // split reduction, or a caller that wants the fp32 sums themselves: accumulators to partial[z][m][co]
        // (row-major like the output; Co % 8 == 0), 16 bytes at a time
        float *part = p.partial + (size_t)split_z * p.M * p.Co;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int m = m0 + wave_m + i * 32 + frag_row;
            if (m >= p.m_end) continue;
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int co = n0 + wave_n + j * 32 + 8 * g4 + 4 * frag_kg;
                    if (co < p.Co)
                        *reinterpret_cast<float4 *>(part + (size_t)m * p.Co + co) =
                            make_float4(acc[i][j][4 * g4], acc[i][j][4 * g4 + 1], acc[i][j][4 * g4 + 2], acc[i][j][4 * g4 + 3]);
                }
        }
        return;
    }
    if ((p.Co & 7) == 0) {
        // Through LDS, one 32-row block of the wave tile at a time, so that global stores are 16 bytes per lane and
        // a row's WN channels leave as one contiguous run.  Staged rows are padded by 16 bytes, and 8-byte unit u of
        // row r sits at u ^ ((r >> 3) % 4): the 32 rows that one 8-byte write instruction covers then fall on 16
        // different bank pairs (two rows each: the least 256 bytes over 128 bytes of banks allow).  A 16-byte chunk c
        // of row r is therefore found at chunk c ^ ((r >> 4) % 2), its halves exchanged when bit 3 of r is set.
        constexpr int CPR = WN / 8;                   // 16-byte chunks per staged row
        constexpr int PW = WN + 8;                    // staged row pitch, elements
        constexpr int RS = 32 * PW;                   // staging elements per wave
        constexpr bool USE_A = SZA >= SZB;
        constexpr int SZ = USE_A ? SZA : SZB;
        constexpr int WPB = SZ / RS;                  // waves whose staging fits one stage buffer
        static_assert(WPB >= 1 && NW <= WPB * NS, "epilogue staging must fit the stage buffers of one operand");
        static_assert((USE_A ? SZB : SZA) * 2 >= BN * 4, "the bias vector must fit a stage buffer of the other operand");
        wait_lgkmcnt0();
        __syncthreads();                              // every wave is done reading operands: LDS is free
        const int bi = wave / WPB;
        bf16_t *stg = bi == 0 ? (USE_A ? sa0 : sb0) : bi == 1 ? (USE_A ? sa1 : sb1) : bi == 2 ? (USE_A ? sa2 : sb2) : (USE_A ? sa3 : sb3);
        stg += (wave % WPB) * RS;
        float *s_bias = reinterpret_cast<float *>(USE_A ? sb0 : sa0);
        const bool has_bias = p.bias != nullptr;
        if (has_bias) {                               // uniform
            if (tid < BN) s_bias[tid] = bias_t;
            __syncthreads();
        }
        // conversion and staging of block (i, *): + bias, ReLU as a 16-bit integer maximum on the rounded pair
        auto stage_block = [&](int i, auto bias_c, auto relu_c) __attribute__((always_inline)) {
            constexpr bool BIAS = decltype(bias_c)::value, RELU = decltype(relu_c)::value;
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    float v0 = acc[i][j][4 * g4], v1 = acc[i][j][4 * g4 + 1], v2 = acc[i][j][4 * g4 + 2], v3 = acc[i][j][4 * g4 + 3];
                    if (BIAS) {
                        const float4 b4 = *reinterpret_cast<const float4 *>(s_bias + wave_n + j * 32 + 8 * g4 + 4 * frag_kg);
                        v0 += b4.x; v1 += b4.y; v2 += b4.z; v3 += b4.w;
                    }
                    uint2 pk = make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
                    if (RELU) {
                        pk.x = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, pk.x), s16x2{0, 0}));
                        pk.y = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, pk.y), s16x2{0, 0}));
                    }
                    *reinterpret_cast<uint2 *>(stg + frag_row * PW + 4 * ((j * 8 + 2 * g4 + frag_kg) ^ ((frag_row >> 3) & 3))) = pk;
                }
        };
        // Common case (output pixel index == GEMM row, no mask, output below 2 GiB, a store instruction covers whole
        // staged rows): one buffer store per 64/CPR rows; rows past the end and columns past Co get an offset the
        // resource rejects, which takes the place of a bounds branch.
        constexpr bool ROWS_PER_STORE_OK = 64 % CPR == 0;
        constexpr int RPI = ROWS_PER_STORE_OK ? 64 / CPR : 1;
        const bool fast_store = ROWS_PER_STORE_OK && p.linear_out && p.mask == nullptr && p.out_bytes != 0;
        const out_rsrc_t rs_out = make_out_rsrc(p.out, p.out_bytes);
        const int st_r = lane / CPR, st_c = lane % CPR;
        auto staged_chunk = [&](int r, int c) __attribute__((always_inline)) {
            const uint4 v = *reinterpret_cast<const uint4 *>(stg + r * PW + ((c ^ ((r >> 4) & 1)) << 3));
            return ((r >> 3) & 1) ? make_uint4(v.z, v.w, v.x, v.y) : v;
        };
        const bool st_col_ok = n0 + wave_n + st_c * 8 < p.Co;
        const unsigned st_lane_off = (unsigned)((st_r * p.Co + n0 + wave_n + st_c * 8) * 2);
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            if (has_bias) { if (p.relu) stage_block(i, std::true_type{}, std::true_type{}); else stage_block(i, std::true_type{}, std::false_type{}); }
            else { if (p.relu) stage_block(i, std::false_type{}, std::true_type{}); else stage_block(i, std::false_type{}, std::false_type{}); }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (fast_store) {
                const int mb = m0 + wave_m + i * 32;
                const unsigned blk_off = (unsigned)mb * (unsigned)(p.Co * 2);   // below 2^32: the output is below 2^31 and a tile adds little
                const int rows_left = p.m_end - mb;
#pragma unroll
                for (int k = 0; k < 32 / RPI; ++k) {
                    const uint4 v = staged_chunk(st_r + k * RPI, st_c);
                    const bool ok = st_col_ok && st_r + k * RPI < rows_left;
                    const unsigned off = ok ? st_lane_off + blk_off + (unsigned)(k * RPI * p.Co * 2) : OOB;
                    if (p.nt_out) buffer_store16_nt(rs_out, off, v);
                    else buffer_store16(rs_out, off, v);
                }
            } else {
#pragma unroll
                for (int k = 0; k < 32 * CPR / 64; ++k) {
                    const int idx = k * 64 + lane;
                    const int r = idx / CPR, c = idx % CPR;
                    const int m = m0 + wave_m + i * 32 + r, co = n0 + wave_n + c * 8;
                    uint4 v = staged_chunk(r, c);
                    if (m < p.m_end && co < p.Co) {
                        const long long off = out_pixel(m) * p.Co + co;
                        if (p.mask != nullptr) {
                            const uint4 mk = *reinterpret_cast<const uint4 *>(p.mask + off);
                            v = make_uint4(mask_bf16x2(v.x, mk.x), mask_bf16x2(v.y, mk.y), mask_bf16x2(v.z, mk.z), mask_bf16x2(v.w, mk.w));
                        }
                        typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
                        const u32x4 vv = {v.x, v.y, v.z, v.w};
                        if (p.nt_out) __builtin_nontemporal_store(vv, reinterpret_cast<u32x4 *>(p.out + off));
                        else *reinterpret_cast<u32x4 *>(p.out + off) = vv;
                    }
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    } else {
        // output channel counts that are not a multiple of 8: element by element
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int m = m0 + wave_m + i * 32 + frag_row;
            if (m >= p.m_end) continue;
            const long long orow = out_pixel(m) * p.Co;
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int co = n0 + wave_n + j * 32 + 8 * (e >> 2) + 4 * frag_kg + (e & 3);
                    if (co < p.Co) {
                        float v = acc[i][j][e] + (p.bias != nullptr ? p.bias[co] : 0.f);
                        if (p.relu) v = fmaxf(v, 0.f);
                        const bool keep = p.mask == nullptr || mask_keeps(p.mask + orow + co);
                        p.out[orow + co] = keep ? f32_to_bf16(v) : (bf16_t)0;
                    }
                }
        }
    }
}

// Launches the tile shape on GEMM rows [m_begin, m_end) of the problem (m_end < 0: to the last row).
template <int BM, int BN, int BKT, int NS, int WR, int WC, bool BT = false>
int launch(IgemmParams p, hipStream_t st, long long m_begin = 0, long long m_end = -1)
{
    static const bool tap_outer_forced = getenv("MXC_TAP_OUTER") != nullptr;   // tuning sweeps only; read once
    const long long M = (long long)p.N * p.Mh * p.Mw;
    if (m_end < 0 || m_end > M) m_end = M;
    if (m_begin >= m_end) return MXC_OK;
    const long long mt = (m_end - m_begin + BM - 1) / BM;
    p.n_tiles = (p.Co + BN - 1) / BN;
    if (mt * p.n_tiles > 0x3FFFFFFFll) return MXC_ERR_SHAPE;
    p.M = (int)M;
    p.m_begin = (int)m_begin;
    p.m_end = (int)m_end;
    p.m_tiles = (int)mt;
    p.in_bytes = (unsigned)((long long)p.N * p.Hi * p.Wi * p.pix * 2);
    p.wm_bytes = BT ? p.bt_w_bytes : (unsigned)((long long)p.Co * p.TR * p.TS * p.Ci * 2);
    // MXC_TAP_OUTER=1 (tuning only) keeps the filter's own order, all channels of a tap before the next tap
    p.tap_inner = (!BT && p.Ci % BKT == 0 && p.TR * p.TS > 1 && !tap_outer_forced) ? 1 : 0;
    p.linear_out = (p.out_mul_h == 1 && p.out_mul_w == 1 && p.out_off_h == 0 && p.out_off_w == 0 && p.Mh == p.Ho && p.Mw == p.Wo) ? 1 : 0;
    // results of a large layer leave as non-temporal stores: the caches keep serving this kernel's operand reads
    static const char *nt_forced = getenv("MXC_NT_OUT");                      // tuning sweeps only; read once
    const long long out_bytes = (long long)p.N * p.Ho * p.Wo * p.Co * 2;
    p.out_bytes = out_bytes < 0x7FFF0000ll ? (unsigned)out_bytes : 0u;
    p.nt_out = nt_forced ? atoi(nt_forced) : ((long long)p.N * p.Ho * p.Wo * p.Co * 2 >= (128ll << 20) ? 1 : 0);
    if (p.splits > 1) {
        // even stage ranges; the last split may be shorter, none is empty
        const int KT = (p.TR * p.TS * p.Ci + BKT - 1) / BKT;
        p.split_stages = (KT + p.splits - 1) / p.splits;
        p.splits = (KT + p.split_stages - 1) / p.split_stages;
        if (!p.linear_out || !p.partial || m_begin != 0 || m_end != M) return MXC_ERR_UNSUPPORTED;
    }
    const long long total = (long long)p.m_tiles * p.n_tiles * (p.splits > 1 ? p.splits : 1);
    if (total > 0x3FFFFFFFll) return MXC_ERR_SHAPE;
    const int grid = (int)((total + 7) / 8) * 8;
    if constexpr (!BT) {
        if (p.tap_inner) {
            hipLaunchKernelGGL((igemm_kernel<BM, BN, BKT, NS, WR, WC, false, true>), dim3((unsigned)grid), dim3(64 * WR * WC), 0, st, p);
            return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
        }
    }
    hipLaunchKernelGGL((igemm_kernel<BM, BN, BKT, NS, WR, WC, BT, false>), dim3((unsigned)grid), dim3(64 * WR * WC), 0, st, p);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

// A tile shape the launcher can pick: output tile, workgroups that fit one CU at a time (LDS and
// register budget) and the matrix-pipe utilisation it reaches relative to the 256x256 tile when the
// chip is full (fitted to per-layer times of the AlexNet- and VGG-style stacks run back to back).
struct TileChoice { int bm, bn, bk, slots; float util; const char *name; };   // bk: reduction elements per stage
const TileChoice kTiles[] = {
    {128, 128, 64, 2, 0.91f, "igemm_128x128_k64s2_w4"},
    {256, 256, 64, 1, 1.15f, "igemm_256x256_k64s2_w8"},
    {256, 128, 64, 1, 0.95f, "igemm_256x128_k64s3_w8"},
    {128, 256, 64, 1, 0.97f, "igemm_128x256_k64s3_w8"},
    {128, 64, 64, 3, 0.65f, "igemm_128x64_k64s2_w4"},
    {256, 64, 32, 2, 0.60f, "igemm_256x64_k32s3_w4"},
    {128, 32, 64, 4, 0.33f, "igemm_128x32_k64s2_w4"},
    {256, 32, 64, 2, 0.33f, "igemm_256x32_k64s2_w4"},
    {256, 192, 64, 1, 1.05f, "igemm_256x192_k64s2_w8"},
    {192, 256, 64, 1, 1.05f, "igemm_192x256_k64s2_w8"},
    {64, 256, 64, 1, 0.55f, "igemm_64x256_k64s3_w8"},
    {64, 128, 64, 2, 0.45f, "igemm_64x128_k64s3_w4"},
    {192, 128, 64, 1, 0.90f, "igemm_192x128_k64s3_w8"},
};
constexpr int N_TILE_CHOICES = sizeof(kTiles) / sizeof(kTiles[0]);
// plan index of the streaming kernel (stream.hip): not a tile of this file's kernel, one launch for all rows
constexpr int STREAM_TILE = N_TILE_CHOICES;
const char *const kStreamName = "igemm_stream";
// ... and of the window kernel (window.hip), likewise
constexpr int WINDOW_TILE = N_TILE_CHOICES + 1;
const char *const kWindowName = "igemm_window";
inline bool whole_launch(int idx) { return idx == STREAM_TILE || idx == WINDOW_TILE; }

// the tiles that also exist reading a 1x1 filter in place (transposed tiles)
bool has_bt(int idx) { return idx == 0 || idx == 1 || idx == 4; }

int launch_choice(int idx, const IgemmParams &p, hipStream_t st, bool bt = false, long long m_begin = 0, long long m_end = -1)
{
    if (bt) {
        switch (idx) {
        case 0: return launch<128, 128, 64, 2, 2, 2, true>(p, st, m_begin, m_end);
        case 1: return launch<256, 256, 64, 2, 2, 4, true>(p, st, m_begin, m_end);
        case 4: return launch<128, 64, 64, 2, 2, 2, true>(p, st, m_begin, m_end);
        default: return MXC_ERR_UNSUPPORTED;
        }
    }
    switch (idx) {
    case 0: return launch<128, 128, 64, 2, 2, 2>(p, st, m_begin, m_end);
    case 1: return launch<256, 256, 64, 2, 2, 4>(p, st, m_begin, m_end);
    case 2: return launch<256, 128, 64, 3, 4, 2>(p, st, m_begin, m_end);
    case 3: return launch<128, 256, 64, 3, 2, 4>(p, st, m_begin, m_end);
    case 4: return launch<128, 64, 64, 2, 2, 2>(p, st, m_begin, m_end);
    case 5: return launch<256, 64, 32, 3, 4, 1>(p, st, m_begin, m_end);
    case 6: return launch<128, 32, 64, 2, 4, 1>(p, st, m_begin, m_end);
    case 7: return launch<256, 32, 64, 2, 4, 1>(p, st, m_begin, m_end);
    case 8: return launch<256, 192, 64, 2, 4, 2>(p, st, m_begin, m_end);
    case 9: return launch<192, 256, 64, 2, 2, 4>(p, st, m_begin, m_end);
    case 10: return launch<64, 256, 64, 3, 2, 4>(p, st, m_begin, m_end);
    case 11: return launch<64, 128, 64, 3, 2, 2>(p, st, m_begin, m_end);
    default: return launch<192, 128, 64, 3, 2, 4>(p, st, m_begin, m_end);
    }
}

// How a GEMM of M rows is run: every row by tile shape `main`, or - when the last round of main tiles would
// leave most CUs idle - rows [0, rows_main) by `main` in whole rounds over the chip and the rest by a second
// launch of the smaller shape `tail` (tail < 0: one launch).
struct Plan { int main, tail; long long rows_main; };

int tile_index(const char *name, size_t len)
{
    for (int i = 0; i < N_TILE_CHOICES; ++i)
        if (strlen(kTiles[i].name) == len && !strncmp(name, kTiles[i].name, len)) return i;
    if (strlen(kStreamName) == len && !strncmp(name, kStreamName, len)) return STREAM_TILE;
    if (strlen(kWindowName) == len && !strncmp(name, kWindowName, len)) return WINDOW_TILE;
    return -1;
}

// rows covered by the whole rounds of shape t over the chip's workgroup slots
long long whole_round_rows(const TileChoice &t, long long M, int Co)
{
    const long long n_tiles = (Co + t.bn - 1) / t.bn, slots = 256LL * t.slots;
    const long long tiles = ((M + t.bm - 1) / t.bm) * n_tiles;
    const long long rows = (tiles / slots) * slots / n_tiles * t.bm;
    return rows < M ? rows : M;
}

// Modelled time of shape t on M rows.  Tiles are dealt evenly to the 256 CUs, so a CU works through
// ceil(tiles/256) tiles, `slots` at a time; a tile costs its area over the utilisation the shape reaches,
// which drops when fewer workgroups than `slots` share the CU (less latency hiding).  Padding waste and the
// partly filled last round are what differ between shapes.
double model_time(const TileChoice &t, long long M, int Co, int KT, double fixed)
{
    const long long tiles = ((M + t.bm - 1) / t.bm) * ((Co + t.bn - 1) / t.bn);
    const long long per_cu = (tiles + 255) / 256;
    const double resident = per_cu < t.slots ? (double)per_cu : (double)t.slots;
    const double util = t.util * (0.6 + 0.4 * resident / t.slots);
    return (double)per_cu * ((double)t.bm * t.bn / util * KT + fixed / resident);
}

#include "tuned_igemm.inc"

// Plan choice, in this order: MXC_FORCE_VARIANT=<name> or <main>+<tail> (tuning sweeps only); the table of
// measured best plans (tuned_igemm.inc, written by the tuning script from timings on the device) when it
// holds this GEMM; else the least modelled time over single shapes and main+tail pairs.
// allow_stream = false: callers that need a tile of this file's kernel, not one of the whole-launch kernels (split
// reductions, in-place filters).
thread_local long long g_key_M = 0;
thread_local int g_key_Co = 0, g_key_Kd = 0;

Plan choose_plan(long long M, int Co, int Kd, bool allow_stream = true)
{
    g_key_M = M; g_key_Co = Co; g_key_Kd = Kd;
    if (const char *f = getenv("MXC_FORCE_VARIANT")) {
        const char *plus = strchr(f, '+');
        const int a = tile_index(f, plus ? (size_t)(plus - f) : strlen(f));
        const int b = plus ? tile_index(plus + 1, strlen(plus + 1)) : -1;
        if (a >= 0 && whole_launch(a) && !plus && allow_stream) return Plan{a, -1, M};
        if (a >= 0 && !whole_launch(a) && !whole_launch(b) && (!plus || b >= 0)) {
            const long long rows = b >= 0 ? whole_round_rows(kTiles[a], M, Co) : M;
            return (b >= 0 && rows > 0 && rows < M) ? Plan{a, b, rows} : Plan{a, -1, M};
        }
    }
    for (const TunedIgemm &e : kTunedIgemm)
        if (e.M == M && e.Co == Co && e.Kd == Kd) {
            const int a = tile_index(e.main, strlen(e.main)), b = e.tail[0] ? tile_index(e.tail, strlen(e.tail)) : -1;
            if (a < 0 || whole_launch(b) || (whole_launch(a) && !allow_stream)) break;
            if (whole_launch(a)) return Plan{a, -1, M};
            const long long rows = b >= 0 ? whole_round_rows(kTiles[a], M, Co) : M;
            return (b >= 0 && rows > 0 && rows < M) ? Plan{a, b, rows} : Plan{a, -1, M};
        }
    // Reductions of one or two stages (first layers): a workgroup's fixed cost (launch, pipeline fill,
    // epilogue: about 4 us, shared by the workgroups resident on the CU) outweighs its matrix work, so
    // fewer, larger tiles win.  In the model's units (tile area x stages at 256x256 speed) that cost
    // is about 150000; a second launch costs about 200000 (5 us of drain, launch and refill).
    const int KT = (Kd + 63) / 64;
    const double fixed = KT <= 2 ? 150000.0 : 0.0, second_launch = 200000.0;
    Plan best{0, -1, M};
    double best_t = 1e300;
    for (int i = 0; i < N_TILE_CHOICES; ++i) {
        const double t1 = model_time(kTiles[i], M, Co, KT, fixed);
        if (t1 < best_t) { best_t = t1; best = Plan{i, -1, M}; }
        const long long rows = whole_round_rows(kTiles[i], M, Co);
        if (rows <= 0 || rows >= M) continue;
        const double t_main = model_time(kTiles[i], rows, Co, KT, fixed);
        for (int j = 0; j < N_TILE_CHOICES; ++j) {
            if (j == i) continue;
            const double t2 = t_main + model_time(kTiles[j], M - rows, Co, KT, fixed) + second_launch;
            if (t2 < best_t) { best_t = t2; best = Plan{i, j, rows}; }
        }
    }
    return best;
}

int choose_tile(long long M, int Co, int Kd) { return choose_plan(M, Co, Kd, false).main; }

// the plan for one launch site: the streaming or the window kernel only where it can run the problem
Plan plan_for(const IgemmParams &p, long long M, int Co, int Kd, bool tiles_only = false)
{
    const Plan pl = choose_plan(M, Co, Kd, !tiles_only);
    if (pl.main == STREAM_TILE && !stream_applicable(p)) return choose_plan(M, Co, Kd, false);
    if (pl.main == WINDOW_TILE && !window_applicable(p)) return choose_plan(M, Co, Kd, false);
    return pl;
}

// runs the plan: one or two launches on the stream
int launch_plan(const Plan &pl, const IgemmParams &p, hipStream_t st, bool bt = false)
{
    if (pl.main == STREAM_TILE) return stream_launch(p, st);
    if (pl.main == WINDOW_TILE) return window_launch(p, st);
    if (pl.tail < 0) return launch_choice(pl.main, p, st, bt);
    const int rc = launch_choice(pl.main, p, st, bt, 0, pl.rows_main);
    if (rc != MXC_OK) return rc;
    return launch_choice(pl.tail, p, st, bt, pl.rows_main, -1);
}

// name of a plan for mxc_last_variant(): "<main>" or "<main>+<tail>"
const char *plan_name(const Plan &pl)
{
    static thread_local char name[96];
    if (pl.main == STREAM_TILE) return kStreamName;
    if (pl.main == WINDOW_TILE) return kWindowName;
    if (pl.tail < 0) return kTiles[pl.main].name;
    snprintf(name, sizeof(name), "%s+%s", kTiles[pl.main].name, kTiles[pl.tail].name);
    return name;
}

// The kernel addresses both operands with signed 32-bit byte offsets, packs tile-row coordinates
// into 16 bits and holds at most MAX_TAPS filter taps in its tap table.
bool igemm_dims_ok(long long in_elems, long long wm_elems, long long M, int Hi, int Wi, int span, int taps)
{
    return in_elems * 2 < 0x7FFF0000ll && wm_elems * 2 < 0x7FFF0000ll && M < 0x7FFFFFFFll && Hi + span <= 8192 &&
           Wi + span <= 8192 && taps <= MAX_TAPS;
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

// dx[n][h_first + stride*a][v_first + stride*b][:] = 0 for the Mh x Mw pixels of one residue class;
// one thread per cw consecutive channels (cw = 8: one 16-byte store).
__global__ __launch_bounds__(256) void zero_phase_kernel(bf16_t *__restrict__ dx, long long n_thr, int H, int W, int C, int cw,
                                                         int stride, int h_first, int v_first, int Mh, int Mw)
{
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= n_thr) return;
    const int per_pix = C / cw;
    const int ch = (int)(gid % per_pix) * cw;
    long long t = gid / per_pix;
    const int b = (int)(t % Mw); t /= Mw;
    const int a = (int)(t % Mh);
    const long long n = t / Mh;
    bf16_t *d = dx + ((n * H + (h_first + stride * a)) * W + (v_first + stride * b)) * C + ch;
    if (cw == 8) *reinterpret_cast<uint4 *>(d) = make_uint4(0, 0, 0, 0);
    else *d = 0;
}

}  // namespace

namespace {

// How many ways to split the reduction of a GEMM whose tiles would leave most of the chip idle
// (FullyConnected-shaped and small-batch problems): enough workgroups to fill the slots, at least 8
// stages per split, at most 32 splits.  1 = no split (every layer of the benchmark stacks).
int split_count(long long M, int Co, int Kd)
{
    const TileChoice &t = kTiles[choose_tile(M, Co, Kd)];
    const long long tiles = ((M + t.bm - 1) / t.bm) * ((Co + t.bn - 1) / t.bn);
    const long long slots = 256LL * t.slots;
    if (tiles * 2 > slots) return 1;
    long long sp = slots / tiles;
    const long long KT = (Kd + 63) / 64;
    if (sp > KT / 8) sp = KT / 8;
    if (sp > 32) sp = 32;
    return sp >= 2 ? (int)sp : 1;
}

// out[m][co] = act(sum_z partial[z][m][co] + bias[co]) in ascending z (fixed order), 4 columns per thread
__global__ __launch_bounds__(256) void split_finish_kernel(const float *__restrict__ partial, bf16_t *__restrict__ out, long long MC,
                                                           int Co, int splits, const float *__restrict__ bias, int relu,
                                                           const bf16_t *__restrict__ mask)
{
    const long long i4 = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i4 >= MC) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int z = 0; z < splits; ++z) {
        const float4 v = *reinterpret_cast<const float4 *>(partial + (size_t)z * MC + i4);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    if (bias != nullptr) {
        const int co = (int)(i4 % Co);          // Co % 8 == 0: the four columns share a row
        acc.x += bias[co]; acc.y += bias[co + 1]; acc.z += bias[co + 2]; acc.w += bias[co + 3];
    }
    if (relu) { acc.x = fmaxf(acc.x, 0.f); acc.y = fmaxf(acc.y, 0.f); acc.z = fmaxf(acc.z, 0.f); acc.w = fmaxf(acc.w, 0.f); }
    uint2 o = make_uint2((uint32_t)f32_to_bf16(acc.x) | ((uint32_t)f32_to_bf16(acc.y) << 16),
                         (uint32_t)f32_to_bf16(acc.z) | ((uint32_t)f32_to_bf16(acc.w) << 16));
    if (mask != nullptr) {
        const uint2 mk = *reinterpret_cast<const uint2 *>(mask + i4);
        o = make_uint2(mask_bf16x2(o.x, mk.x), mask_bf16x2(o.y, mk.y));
    }
    *reinterpret_cast<uint2 *>(out + i4) = o;
}

// One GEMM (output pixels numbered like the GEMM rows, Co % 8 == 0) run as `sp` splits of the reduction
// plus the finishing kernel, which applies `post`.
int launch_split(int tc, IgemmParams p, long long M, int sp, void *split_ws, void *out, const PostOp &post, hipStream_t st,
                 const char **variant, bool bt = false)
{
    p.splits = sp;
    p.partial = (float *)split_ws;
    p.bias = nullptr; p.relu = 0; p.mask = nullptr;      // applied by the finishing kernel
    const int rc = launch_choice(tc, p, st, bt);
    if (rc != MXC_OK) return rc;
    const long long MC = M * p.Co;
    if ((MC / 4 + 255) / 256 > 0x7FFFFFFFll) return MXC_ERR_SHAPE;
    // the launcher evens out the stage ranges, which can lower the split count: recompute it the same way
    const int bk = kTiles[tc].bk;
    const int KT = (p.TR * p.TS * p.Ci + bk - 1) / bk, per = (KT + sp - 1) / sp, used = (KT + per - 1) / per;
    static thread_local char split_name[64];
    snprintf(split_name, sizeof(split_name), "%s%s_split%d", kTiles[tc].name, bt ? "_inplace" : "", used);
    *variant = split_name;
    hipLaunchKernelGGL(split_finish_kernel, dim3((unsigned)((MC / 4 + 255) / 256)), dim3(256), 0, st, (const float *)split_ws,
                       (bf16_t *)out, MC, p.Co, used, post.bias, post.relu, (const bf16_t *)post.mask);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

}  // namespace

const char *igemm_tile_name(int index) { return index >= 0 && index < N_TILE_CHOICES ? kTiles[index].name : nullptr; }
const char *igemm_stream_name(int index) { return index == 0 ? kStreamName : index == 1 ? kWindowName : nullptr; }
void igemm_last_plan_key(long long *M, int *Co, int *Kd) { *M = g_key_M; *Co = g_key_Co; *Kd = g_key_Kd; }

size_t igemm_bwd_data_split_bytes(const ConvShape &s)
{
    if (s.stride != 1 || s.C % 8 != 0) return 0;       // one residue class, output numbered like the GEMM rows
    const long long M = (long long)s.N * s.H * s.W;
    const int sp = split_count(M, s.C, s.R * s.S * s.K);
    return sp > 1 ? (size_t)sp * M * s.C * sizeof(float) : 0;
}

size_t igemm_fwd_split_bytes(const ConvShape &s)
{
    if (s.K % 8 != 0) return 0;
    const long long M = (long long)s.N * s.P * s.Q;
    const int sp = split_count(M, s.K, s.R * s.S * s.C);
    return sp > 1 ? (size_t)sp * M * s.K * sizeof(float) : 0;
}

bool igemm_fwd_supported(const ConvShape &s)
{
    return s.C % 8 == 0 && igemm_dims_ok((long long)s.N * s.H * s.W * s.C, (long long)s.K * s.R * s.S * s.C,
                                         (long long)s.N * s.P * s.Q, s.H, s.W, s.pad + s.R + s.S + s.stride, s.R * s.S);
}

int igemm_fwd(const ConvShape &s, const void *x, const void *w, void *y, hipStream_t st, const char **variant, const PostOp &post,
              void *split_ws)
{
    IgemmParams p{};
    p.bias = post.bias; p.relu = post.relu;
    p.in = (const bf16_t *)x; p.wm = (const bf16_t *)w; p.out = (bf16_t *)y;
    p.N = s.N; p.Hi = s.H; p.Wi = s.W; p.Ci = s.C; p.pix = s.C; p.Co = s.K;
    p.TR = s.R; p.TS = s.S; p.tstep_h = 1; p.tstep_w = 1;
    p.Mh = s.P; p.Mw = s.Q;
    p.in_mul_h = s.stride; p.in_mul_w = s.stride; p.in_off_h = -s.pad; p.in_off_w = -s.pad;
    p.Ho = s.P; p.Wo = s.Q; p.out_mul_h = 1; p.out_mul_w = 1; p.out_off_h = 0; p.out_off_w = 0;
    const long long M = (long long)s.N * s.P * s.Q;
    const int sp = (split_ws != nullptr && s.K % 8 == 0) ? split_count(M, s.K, s.R * s.S * s.C) : 1;
    const Plan pl = plan_for(p, M, s.K, s.R * s.S * s.C, sp > 1);
    *variant = plan_name(pl);
    if (sp > 1) return launch_split(pl.main, p, M, sp, split_ws, y, post, st, variant);
    return launch_plan(pl, p, st);
}

// Plain GEMM on the same kernels: out[m][n] = sum_k a[m][k] * b[n][k], a and b bf16 (row-major, k contiguous, k % 8 == 0),
// out fp32, n % 8 == 0.  It is the 1x1 convolution of an M-image batch of 1x1 images whose fp32 accumulators are
// stored unrounded (the transform-domain convolution multiplies its 16 planes with it).
bool igemm_gemm_f32_supported(long long M, int Kd, int Nn)
{
    return Kd % 8 == 0 && Nn % 8 == 0 && igemm_dims_ok(M * Kd, (long long)Nn * Kd, M, 1, 1, 4, 1) && M * Nn * 4 < (1ll << 40);
}

int igemm_gemm_f32(long long M, int Kd, int Nn, const void *a, const void *b, float *out, hipStream_t st, const char **variant)
{
    IgemmParams p{};
    p.in = (const bf16_t *)a; p.wm = (const bf16_t *)b; p.out = nullptr;
    p.partial = out; p.f32_out = 1;
    p.N = (int)M; p.Hi = 1; p.Wi = 1; p.Ci = Kd; p.pix = Kd; p.Co = Nn;
    p.TR = 1; p.TS = 1; p.tstep_h = 1; p.tstep_w = 1;
    p.Mh = 1; p.Mw = 1;
    p.in_mul_h = 1; p.in_mul_w = 1; p.in_off_h = 0; p.in_off_w = 0;
    p.Ho = 1; p.Wo = 1; p.out_mul_h = 1; p.out_mul_w = 1; p.out_off_h = 0; p.out_off_w = 0;
    const Plan pl = choose_plan(M, Nn, Kd, false);
    *variant = plan_name(pl);
    return launch_plan(pl, p, st);
}

bool igemm_fwd_smallc_supported(const ConvShape &s)
{
    const SmallCGeom g = smallc_geom(s);
    return s.C <= 4 && igemm_dims_ok((long long)s.N * g.Hp * g.Wp * g.pix, (long long)s.K * s.R * g.run,
                                     (long long)s.N * s.P * s.Q, g.Hp, g.Wp, s.R + s.S + s.stride, s.R);
}

// Forward for a small-C image packed by smallc_pack_x / smallc_pack_w: R taps (filter rows), each a
// contiguous run of S*pix elements of the zero-bordered image.
int igemm_fwd_smallc(const ConvShape &s, const void *xp, const void *wp, void *y, hipStream_t st, const char **variant,
                     const PostOp &post)
{
    const SmallCGeom g = smallc_geom(s);
    IgemmParams p{};
    p.bias = post.bias; p.relu = post.relu;
    p.in = (const bf16_t *)xp; p.wm = (const bf16_t *)wp; p.out = (bf16_t *)y;
    p.N = s.N; p.Hi = g.Hp; p.Wi = g.Wp; p.Ci = g.run; p.pix = g.pix; p.Co = s.K;
    p.TR = s.R; p.TS = 1; p.tstep_h = 1; p.tstep_w = 1;
    p.Mh = s.P; p.Mw = s.Q;
    p.in_mul_h = s.stride; p.in_mul_w = s.stride; p.in_off_h = 0; p.in_off_w = 0;
    p.Ho = s.P; p.Wo = s.Q; p.out_mul_h = 1; p.out_mul_w = 1; p.out_off_h = 0; p.out_off_w = 0;
    const Plan pl = plan_for(p, (long long)s.N * s.P * s.Q, s.K, s.R * g.run);
    *variant = plan_name(pl);
    return launch_plan(pl, p, st);
}

bool igemm_bwd_data_supported(const ConvShape &s)
{
    return s.K % 8 == 0 && s.stride <= 4 &&
           igemm_dims_ok((long long)s.N * s.P * s.Q * s.K, (long long)s.K * s.R * s.S * s.C, (long long)s.N * s.H * s.W, s.P,
                         s.Q, s.pad + s.R + s.S + s.stride, s.R * s.S);
}

size_t igemm_bwd_data_workspace(const ConvShape &s) { return (size_t)s.K * s.R * s.S * s.C * sizeof(bf16_t); }

// A large 1x1 filter at stride 1 (FullyConnected) is read in place, as transposed tiles, when the chosen
// tile has that variant: copying it would cost more than the slower operand fetch.
static bool bwd_data_reads_filter_in_place(const ConvShape &s)
{
    return s.R == 1 && s.S == 1 && s.stride == 1 && s.K % 64 == 0 && (long long)s.K * s.C * 2 >= (4ll << 20) &&
           has_bt(choose_tile((long long)s.N * s.H * s.W, s.C, s.K));
}

int igemm_bwd_data_prepare(const ConvShape &s, const void *w, void *wt, hipStream_t st, bool copy_in_place_filter)
{
    if (bwd_data_reads_filter_in_place(s))
        return copy_in_place_filter ? launch_copy(w, wt, (size_t)s.K * s.C * sizeof(bf16_t), st) : MXC_OK;
    if (s.R == 1 && s.S == 1)
        // 1x1: the single class's matrix [C][K] is the transpose of w[K][C] (tiled transpose through LDS)
        return launch_transpose(w, wt, 1, s.K, s.C, 2, st);
    const int total = s.K * s.R * s.S * s.C;
    hipLaunchKernelGGL(repack_bwd_data_filter_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       (const bf16_t *)w, (bf16_t *)wt, s.K, s.C, s.R, s.S, s.stride);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

// wt: the filter as igemm_bwd_data_prepare left it; w_in_place: the filter the in-place variant reads
// (the caller's KRSC filter, or its copy in wt)
int igemm_bwd_data(const ConvShape &s, const void *dy, const void *w_in_place, void *dx, const void *wt, hipStream_t st,
                   const char **variant, const PostOp &post, void *split_ws)
{
    const bool bt = bwd_data_reads_filter_in_place(s);
    const void *w = w_in_place;
    size_t wt_off = 0;
    Plan pl{0, -1, 0};
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
            p.in = (const bf16_t *)dy; p.wm = bt ? (const bf16_t *)w : (const bf16_t *)wt + wt_off; p.out = (bf16_t *)dx;
            p.mask = (const bf16_t *)post.mask;
            p.bt_w_bytes = (unsigned)((long long)s.K * s.C * 2);
            p.N = s.N; p.Hi = s.P; p.Wi = s.Q; p.Ci = s.K; p.pix = s.K; p.Co = s.C;
            p.TR = TR; p.TS = TS; p.tstep_h = -1; p.tstep_w = -1;
            p.Mh = Mh; p.Mw = Mw;
            p.in_mul_h = 1; p.in_mul_w = 1; p.in_off_h = hh0; p.in_off_w = vv0;
            p.Ho = s.H; p.Wo = s.W; p.out_mul_h = s.stride; p.out_mul_w = s.stride; p.out_off_h = h_first; p.out_off_w = v_first;
            wt_off += (size_t)s.C * TR * TS * s.K;
            if (Mh <= 0 || Mw <= 0) continue;
            if (TR * TS == 0) {
                // no tap reaches this residue class (stride larger than the filter): its pixels are zero
                const int cw = (s.C % 8 == 0) ? 8 : 1;   // elements written per thread
                const long long n_thr = (long long)s.N * Mh * Mw * (s.C / cw);
                if ((n_thr + 255) / 256 > 0x7FFFFFFFll) return MXC_ERR_SHAPE;
                hipLaunchKernelGGL(zero_phase_kernel, dim3((unsigned)((n_thr + 255) / 256)), dim3(256), 0, st, (bf16_t *)dx, n_thr,
                                   s.H, s.W, s.C, cw, s.stride, h_first, v_first, Mh, Mw);
                if (hipGetLastError() != hipSuccess) return MXC_ERR_LAUNCH;
                continue;
            }
            const int sp = (split_ws != nullptr && s.stride == 1 && s.C % 8 == 0)
                               ? split_count((long long)s.N * Mh * Mw, s.C, TR * TS * s.K) : 1;
            pl = plan_for(p, (long long)s.N * Mh * Mw, s.C, TR * TS * s.K, bt || sp > 1);
            if (bt && !has_bt(pl.tail)) pl = Plan{pl.main, -1, 0};
            if (sp > 1) return launch_split(pl.main, p, (long long)s.N * Mh * Mw, sp, split_ws, dx, post, st, variant, bt);
            const int rc = launch_plan(pl, p, st, bt);
            if (rc != MXC_OK) return rc;
        }
    }
    *variant = plan_name(pl);
    return MXC_OK;
}

// ---- backward-data for small C (first layers) ------------------------------------------------
// With C <= 4 output channels the GEMM's N dimension would be almost empty.  Instead G consecutive
// output columns form one GEMM row: N' = G*4 (channels padded to 4), and the reduction runs over the
// U columns of dy that reach any of the G pixels.  Per residue class ph of (h+pad) mod stride:
//     dx4[n][h][b*G+g][c] = sum_{j,u,k} dy[n][hh-j][b*G/stride + uoff + u][k] * W2[(g,c)][(j,u,k)]
//     W2[(g,c)][(j,u,k)]  = w[k][ph+stride*j][s][c],  s = g + pad - stride*(u + uoff), zero if s outside [0,S)
// dx4 is then compacted to the caller's C channels.

namespace {

struct SmallCBwd { int G, U, uoff, Wg; };

SmallCBwd smallc_bwd_geom(const ConvShape &s)
{
    SmallCBwd g;
    g.G = 8;
    // floor((pad - S + 1) / stride)
    const int num = s.pad - s.S + 1;
    g.uoff = num >= 0 ? num / s.stride : -((-num + s.stride - 1) / s.stride);
    g.U = (g.G - 1 + s.pad) / s.stride - g.uoff + 1;
    g.Wg = (s.W + g.G - 1) / g.G;
    return g;
}

// all residue classes one after another; class ph holds [G*4][TR_ph*U*K]
__global__ __launch_bounds__(256) void smallc_bwd_pack_w_kernel(const bf16_t *__restrict__ w, bf16_t *__restrict__ w2, int K,
                                                               int C, int R, int S, int stride, int pad, int G, int U,
                                                               int uoff)
{
    const int rows = G * 4;
    int gid = blockIdx.x * blockDim.x + threadIdx.x;
    int ph = 0, TRp = 0;
    for (; ph < stride; ++ph) {
        TRp = ph < R ? (R - ph + stride - 1) / stride : 0;
        const int sz = rows * TRp * U * K;
        if (gid < sz) break;
        gid -= sz;
    }
    if (ph == stride) return;
    // reduction order (u, j, k): the row taps of one dy column are consecutive stages, so the dy row a
    // GEMM row reads at row tap j is the one its neighbour one image row down reads at j+1, one stage
    // later, while it is still in the L2 (with j outermost the reuse came 10 stages later and missed)
    const int k = gid % K; int t = gid / K;
    const int j = t % TRp; t /= TRp;
    const int u = t % U; t /= U;
    const int c = t & 3, g = t >> 2;
    const int r = ph + stride * j;
    const int sidx = g + pad - stride * (u + uoff);
    bf16_t v = 0;
    if (c < C && sidx >= 0 && sidx < S) v = w[(((size_t)k * R + r) * S + sidx) * C + c];
    const size_t phase_base = (size_t)(blockIdx.x * blockDim.x + threadIdx.x) - gid;
    w2[phase_base + gid] = v;
}

// dx[n][h][w][c] = dx4[n][h][w][c], c < C; dx4 rows are Wg*G pixels wide
__global__ __launch_bounds__(256) void smallc_compact_kernel(const uint2 *__restrict__ dx4, bf16_t *__restrict__ dx, long long rows,
                                                            int W, int W4, int C, const bf16_t *__restrict__ mask)
{
    const long long total = rows * W;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const long long row = gid / W;
    const int wv = (int)(gid % W);
    const uint2 v = dx4[row * W4 + wv];
    bf16_t *d = dx + gid * C;
    const bf16_t e[4] = {(bf16_t)(v.x & 0xFFFF), (bf16_t)(v.x >> 16), (bf16_t)(v.y & 0xFFFF), (bf16_t)(v.y >> 16)};
#pragma unroll
    for (int c = 0; c < 4; ++c)
        if (c < C) d[c] = (mask == nullptr || mask_keeps(mask + gid * C + c)) ? e[c] : (bf16_t)0;
}

}  // namespace

bool igemm_bwd_data_smallc_supported(const ConvShape &s)
{
    const SmallCBwd g = smallc_bwd_geom(s);
    return s.C <= 4 && s.K % 8 == 0 && (s.stride == 1 || s.stride == 2 || s.stride == 4) &&
           igemm_dims_ok((long long)s.N * s.P * s.Q * s.K, (long long)g.G * 4 * s.R * g.U * s.K, (long long)s.N * s.H * g.Wg, s.P,
                         s.Q, s.pad + s.R + s.S + s.stride + g.U, s.R * g.U) &&
           (long long)s.N * s.H * g.Wg * g.G * 4 * 2 < 0x7FFF0000ll;
}

void igemm_bwd_data_smallc_workspace(const ConvShape &s, size_t *w2_bytes, size_t *dx4_bytes)
{
    const SmallCBwd g = smallc_bwd_geom(s);
    size_t taps = 0;
    for (int ph = 0; ph < s.stride; ++ph) taps += ph < s.R ? (s.R - ph + s.stride - 1) / s.stride : 0;
    *w2_bytes = (size_t)g.G * 4 * taps * g.U * s.K * 2;
    *dx4_bytes = (size_t)s.N * s.H * g.Wg * g.G * 4 * 2;
}

int igemm_bwd_data_smallc_prepare(const ConvShape &s, const void *w, void *w2, hipStream_t st)
{
    const SmallCBwd g = smallc_bwd_geom(s);
    size_t w2_bytes, dx4_bytes;
    igemm_bwd_data_smallc_workspace(s, &w2_bytes, &dx4_bytes);
    const int total = (int)(w2_bytes / 2);
    hipLaunchKernelGGL(smallc_bwd_pack_w_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, (const bf16_t *)w,
                       (bf16_t *)w2, s.K, s.C, s.R, s.S, s.stride, s.pad, g.G, g.U, g.uoff);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

// w2: the filter as igemm_bwd_data_smallc_prepare packed it
int igemm_bwd_data_smallc(const ConvShape &s, const void *dy, const void *w2, void *dx, void *dx4, hipStream_t st,
                          const char **variant, const PostOp &post)
{
    const SmallCBwd g = smallc_bwd_geom(s);
    size_t w2_off = 0;
    Plan pl{0, -1, 0};
    for (int ph = 0; ph < s.stride; ++ph) {
        const int TR = ph < s.R ? (s.R - ph + s.stride - 1) / s.stride : 0;
        const int hh0 = ph >= s.pad ? 0 : (s.pad - ph + s.stride - 1) / s.stride;
        const int h_first = ph - s.pad + s.stride * hh0;
        const int Mh = h_first < s.H ? (s.H - 1 - h_first) / s.stride + 1 : 0;
        IgemmParams p{};
        p.in = (const bf16_t *)dy; p.wm = (const bf16_t *)w2 + w2_off; p.out = (bf16_t *)dx4;
        p.N = s.N; p.Hi = s.P; p.Wi = s.Q; p.Ci = s.K; p.pix = s.K; p.Co = g.G * 4;
        p.TR = TR; p.TS = g.U; p.tstep_h = -1; p.tstep_w = 1; p.tap_row_inner = 1;
        p.Mh = Mh; p.Mw = g.Wg;
        p.in_mul_h = 1; p.in_mul_w = g.G / s.stride; p.in_off_h = hh0; p.in_off_w = g.uoff;
        p.Ho = s.H; p.Wo = g.Wg; p.out_mul_h = s.stride; p.out_mul_w = 1; p.out_off_h = h_first; p.out_off_w = 0;
        w2_off += (size_t)g.G * 4 * TR * g.U * s.K;
        if (Mh <= 0) continue;
        pl = plan_for(p, (long long)s.N * Mh * g.Wg, p.Co, TR * g.U * s.K);
        const int rc = launch_plan(pl, p, st);
        if (rc != MXC_OK) return rc;
    }
    const long long rows = (long long)s.N * s.H;
    const long long blocks = (rows * s.W + 255) / 256;
    if (blocks > 0x7FFFFFFFll) return MXC_ERR_SHAPE;
    hipLaunchKernelGGL(smallc_compact_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const uint2 *)dx4, (bf16_t *)dx, rows,
                       s.W, g.Wg * g.G, s.C, (const bf16_t *)post.mask);
    *variant = plan_name(pl);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

}  // namespace mxc
