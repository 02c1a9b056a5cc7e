// Streaming implicit GEMM for short reductions: the memory-bound layers.
//
// Same GEMM as igemm.hip,  Out[m][co] = sum_{t,ci} In[pixel(m) + tap(t)][ci] * Wm[co][t*Ci + ci],  for the
// layers whose filter matrix is small (1x1 layers, first layers, K <= 128 with a few hundred reduction
// elements): there the work per output tile is a handful of stages, and a kernel that starts, fills its
// pipeline and drains once per tile spends most of its time doing that instead of moving bytes.  Here
//   * the filter matrix of the workgroup's column tile stays RESIDENT in LDS for the kernel's lifetime;
//   * workgroups are PERSISTENT: each owns a contiguous range of GEMM rows (all ranges equal, so every
//     workgroup moves the same number of bytes) and walks it tile by tile, and the ring of activation stages
//     keeps running across tile boundaries: loads of the next tile are in flight while this one is multiplied
//     and stored;
//   * waves are SPECIALISED: loader waves issue the asynchronous global->LDS loads of the ring and nothing
//     else, compute waves read operands, run the MFMAs and store results.  Loads and stores then never share
//     a wave's memory counter, which matters because a counter that holds both kinds can only be waited on
//     to zero (they complete out of order with respect to each other), and that would empty the ring at every
//     tile end.
// One workgroup barrier per stage hands a landed stage to the compute waves and a consumed slot back to the
// loaders.  Compute wave v owns rows 32v..32v+31 of the row tile and all BN columns (v_mfma_f32_32x32x16_bf16,
// fp32 accumulators, which start from the bias); results leave through a per-wave LDS staging area as 16-byte
// stores, with the same optional ReLU / mask as the other kernel.
#include <type_traits>

#include "mxc_internal.h"

namespace mxc {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

constexpr unsigned OOB = 0x80000000u;   // a buffer offset no operand reaches: the load returns zeros
constexpr int BK = 64;                  // reduction elements per stage

template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ void wait_lgkmcnt0() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void wg_barrier()
{
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
}

struct StreamParams {
    IgemmParams g;
    int KT;          // stages per tile = ceil(T*Ci / 64)
    int n_wg_m;      // workgroups per column tile; workgroup w of them owns rows [m_begin + w*rows_per_wg, + rows_per_wg)
    int rows_per_wg; // a multiple of 32
    int units;       // n_wg_m * n_tiles (the grid is rounded up to whole XCD rounds)
    int per_xcd;     // units per XCD, a multiple of n_tiles
    int b_bytes;     // LDS bytes of the resident filter tile: BN * KT * 128
    int nt;          // bit 0: results leave as non-temporal stores, bit 1: activations arrive as non-temporal loads
    unsigned out_bytes;   // size of the output tensor (< 2^31)
    int d_n, d_a, d_b;   // one row tile further = d_n images + d_a rows + d_b columns of the output grid (d_a < Mh, d_b < Mw)
};

// NC compute waves (row tile BM = 32*NC), NL loader waves, column tile BN (32, 64 or 128), NS ring stages.
// Dynamic LDS: [filter BN x KT*64][ring NS x BM x 64][staging NC x 32 x min(BN,64)][tap table][bias BN].
template <int NC, int NL, int BN, int NS>
__global__ __launch_bounds__(64 * (NC + NL)) void stream_kernel(const StreamParams sp)
{
    const IgemmParams &p = sp.g;
    constexpr int BM = 32 * NC, NW = NC + NL;
    constexpr int NI = BN / 32;
    constexpr int A_LD = BM / 8 / NL;               // wave-wide loads per loader wave per stage (8 tile rows each)
    constexpr int STG_A = BM * BK;                  // elements per ring stage
    constexpr int EW = BN < 64 ? BN : 64;           // staging width (columns)
    static_assert(BM % (8 * NL) == 0 && NL % 2 == 0, "loader split");
    static_assert(NS >= 3 && A_LD * (NS - 1) < 64, "ring depth against the range of the load counter");

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    bf16_t *sB = reinterpret_cast<bf16_t *>(smem);
    bf16_t *sA = reinterpret_cast<bf16_t *>(smem + sp.b_bytes);
    bf16_t *sE = sA + NS * STG_A;
    int2 *tap_tab = reinterpret_cast<int2 *>(sE + NC * 32 * EW);
    float *sBias = reinterpret_cast<float *>(tap_tab + MAX_TAPS + 1);   // BN values: the bias of this column tile, or zeros

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave >= NC;

    // Workgroup -> (row range, column tile).  Consecutive workgroup ids are dealt round-robin to the 8 XCDs;
    // the column tiles of one row range get ids of the same XCD, so the activations they share meet in one L2.
    const int unit = (blockIdx.x & 7) * sp.per_xcd + (blockIdx.x >> 3);
    if (unit >= sp.units) return;
    const int n_tile = unit % p.n_tiles, wg_m = unit / p.n_tiles;
    const int n0 = n_tile * BN;
    const int wg_lo = p.m_begin + wg_m * sp.rows_per_wg;
    const int wg_hi = min(p.m_end, wg_lo + sp.rows_per_wg);   // M < 2^31 - 2^16: no overflow
    const int my_tiles = wg_hi > wg_lo ? (wg_hi - wg_lo + BM - 1) / BM : 0;
    const int KT = sp.KT;
    const int total = my_tiles * KT;                // stages this workgroup runs
    const int T = p.TR * p.TS;
    const int Kd = T * p.Ci;

    // ---- tap table (as in the other kernel; entry T is a sentinel no pixel satisfies) -------------------
    for (int t = tid; t <= T; t += 64 * NW) {
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

    for (int c = tid; c < BN; c += 64 * NW) sBias[c] = (p.bias != nullptr && n0 + c < p.Co) ? p.bias[n0 + c] : 0.f;

    const buf_rsrc_t rs_in = make_buf_rsrc(p.in, p.in_bytes);
    const buf_rsrc_t rs_wm = make_buf_rsrc(p.wm, p.wm_bytes);

    // ---- resident filter: every wave fetches its share once.  Row r, 16-byte chunk c of stage kt lives at
    // chunk position c ^ ((r/2) % 8) of that row (the swizzle the operand reads below undo).
    {
        const int per_stage = BN / 8;               // wave-wide loads per stage (8 rows each)
        for (int idx = wave; idx < KT * per_stage; idx += NW) {
            const int kt = idx / per_stage, i = idx % per_stage;
            const int r = 8 * i + (lane >> 3);
            const int c = (lane & 7) ^ ((r >> 1) & 7);
            const int kd = kt * BK + c * 8;
            const unsigned off = (n0 + r < p.Co && kd < Kd) ? (unsigned)(n0 + r) * (unsigned)(Kd * 2) + (unsigned)kd * 2u : OOB;
            lds_dma16(rs_wm, off, sB + (size_t)kt * BN * BK + i * 8 * BK);
        }
    }
    __syncthreads();        // tap table visible (the filter loads stay in flight)

    if (loader) {
        // =============================== loader waves ===================================================
        const int l = wave - NC;
        const int ld_sub = lane >> 3;
        // wave-wide load i of this wave covers tile rows 8*(l + NL*i) .. +7; NL is even, so the swizzle term
        // (row/2) % 8 = (4*l + lane/16) % 8 is the same for all of them: one reduction offset per lane
        const int ld_chunk = (lane & 7) ^ ((4 * l + (lane >> 4)) & 7);
        const int kq = BK / p.Ci, kr2 = (BK % p.Ci) * 2, Ci2 = p.Ci * 2, Kd2 = Kd * 2;
        const int lim_hw = ((p.Hi - 1) & 0xFFFF) | ((p.Wi - 1) << 16);
        const int kd0 = ld_chunk * 8;
        int a_off[A_LD], a_hw[A_LD];
        int kd2 = 0, ci2 = 0, tap = 0;              // reduction position of this lane's chunk in the cursor's stage
        int pf_kt = 0;                              // prefetch cursor: stage of its tile that is requested next

        // Row bookkeeping.  Row i of this lane sits at output-grid position (image, a, b); the next tile's row is BM
        // GEMM rows further on, BM = d_n images + d_a grid rows + d_b grid columns, so positions and byte offsets
        // advance by additions and two wrap tests - no division after the first tile.
        int row_a[A_LD], row_b[A_LD];
        unsigned row_off[A_LD];                     // byte offset of the row's tap-0 pixel (wraps below zero in the padding)
        int tile_m0 = wg_lo;                        // first GEMM row of the cursor's tile
        const unsigned col_step = (unsigned)(p.in_mul_w * p.pix * 2), row_step = (unsigned)(p.in_mul_h * p.Wi * p.pix * 2);
        const unsigned img_step = (unsigned)(p.Hi * p.Wi * p.pix * 2);
        const unsigned tile_step = (unsigned)sp.d_n * img_step + (unsigned)sp.d_a * row_step + (unsigned)sp.d_b * col_step;
        const unsigned wrap_b = row_step - (unsigned)p.Mw * col_step, wrap_a = img_step - (unsigned)p.Mh * row_step;
        auto publish_rows = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                const int m = tile_m0 + 8 * (l + NL * i) + ld_sub;
                const int h = row_a[i] * p.in_mul_h + p.in_off_h, w = row_b[i] * p.in_mul_w + p.in_off_w;
                a_off[i] = (int)row_off[i];
                a_hw[i] = m < wg_hi ? ((h & 0xFFFF) | (w << 16)) : ((-16384) & 0xFFFF);
            }
            kd2 = kd0 * 2;
            ci2 = (kd0 % p.Ci) * 2;
            tap = kd0 / p.Ci;
        };
        auto first_tile_rows = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                const int m = tile_m0 + 8 * (l + NL * i) + ld_sub;
                const unsigned b = (unsigned)m % (unsigned)p.Mw, t2 = (unsigned)m / (unsigned)p.Mw;
                const unsigned a = t2 % (unsigned)p.Mh, n = t2 / (unsigned)p.Mh;
                const int h = (int)a * p.in_mul_h + p.in_off_h, w = (int)b * p.in_mul_w + p.in_off_w;
                row_a[i] = (int)a;
                row_b[i] = (int)b;
                row_off[i] = (unsigned)((((long long)n * p.Hi + h) * p.Wi + w) * p.pix * 2);
            }
            publish_rows();
        };
        auto next_tile_rows = [&]() __attribute__((always_inline)) {
            tile_m0 += BM;
#pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                int a = row_a[i] + sp.d_a, b = row_b[i] + sp.d_b;
                unsigned off = row_off[i] + tile_step;
                const bool cb = b >= p.Mw;
                b -= cb ? p.Mw : 0;
                a += cb ? 1 : 0;
                off += cb ? wrap_b : 0u;
                const bool ca = a >= p.Mh;
                a -= ca ? p.Mh : 0;
                off += ca ? wrap_a : 0u;
                row_a[i] = a;
                row_b[i] = b;
                row_off[i] = off;
            }
            publish_rows();
        };
        // request the cursor's stage into ring slot `slot`, then advance the cursor
        auto request = [&](int slot) __attribute__((always_inline)) {
            const int2 te = tap_tab[(tap < T && kd2 < Kd2) ? tap : T];
            bf16_t *dst = sA + slot * STG_A;
#pragma unroll
            for (int i = 0; i < A_LD; ++i) {
                const s16x2 hw = __builtin_bit_cast(s16x2, a_hw[i]) + __builtin_bit_cast(s16x2, te.y);
                const s16x2 d = __builtin_bit_cast(s16x2, lim_hw) - hw;
                const int bad = (__builtin_bit_cast(int, hw) | __builtin_bit_cast(int, d)) & (int)0x80008000;
                const unsigned va = bad == 0 ? (unsigned)(a_off[i] + te.x + ci2) : OOB;
                if (sp.nt & 2) lds_dma16_nt(rs_in, va, dst + (l + NL * i) * 8 * BK);
                else lds_dma16(rs_in, va, dst + (l + NL * i) * 8 * BK);
            }
            if (++pf_kt == KT) {
                pf_kt = 0;
                next_tile_rows();
            } else {
                kd2 += BK * 2;
                ci2 += kr2;
                const int carry = ci2 >= Ci2 ? 1 : 0;
                ci2 -= carry ? Ci2 : 0;
                tap += kq + carry;
            }
        };

        first_tile_rows();
#pragma unroll
        for (int s = 0; s < NS; ++s) request(s);
        wait_vmcnt<A_LD * (NS - 1)>();              // the filter share and stage 0 have landed
        wg_barrier();
        int slot = 0;
        for (int g = 0; g < total; ++g) {
            wait_vmcnt<A_LD * (NS - 2)>();          // stage g+1 has landed
            wg_barrier();                           // ... and every compute wave is done with stage g
            request(slot);                          // stage g+NS into the freed slot
            slot = slot + 1 == NS ? 0 : slot + 1;
        }
        wait_vmcnt<0>();                            // drain the requests past the end
        return;
    }

    // ================================= compute waves =======================================================
    // The product is formed transposed, D[co][pixel] (filter fragment as the first MFMA operand): accumulator
    // element e of a 32x32 block then belongs to pixel lane%32 and output column 8*(e/4) + 4*(lane/32) + e%4, so a
    // lane holds runs of four neighbouring columns of one pixel - they convert two at a time
    // (v_cvt_pk_bf16_f32) and go to the staging area eight bytes at a time.
    const int frag_row = lane & 31, frag_kg = lane >> 5;
    const int frag_swz = (frag_row >> 1) & 7;
    const bf16_t *a_base = sA + (wave * 32 + frag_row) * BK;
    const bf16_t *b_base = sB + frag_row * BK;
    bf16_t *stg = sE + wave * 32 * EW;
    // Staging layout: a row holds CPR 16-byte chunks; chunk c of row r sits at position c ^ ((r >> LB) % CPR) and
    // its two 8-byte halves change places when bit 3 of r is set.  The 32 rows that one 8-byte write instruction
    // covers then fall on 16 different bank pairs (two rows each: the least 256 bytes over 128 bytes of banks allow).
    constexpr int CPR = EW / 8;
    constexpr int LB = EW == 64 ? 0 : 1;            // log2 of the rows that share one 128-byte line of banks
    auto stg_chunk = [](int r, int c) __attribute__((always_inline)) { return (c ^ ((r >> LB) & (CPR - 1))) << 3; };
    auto swap_halves = [](uint4 v, bool sw) __attribute__((always_inline)) { return sw ? make_uint4(v.z, v.w, v.x, v.y) : v; };
    constexpr int JN = EW / 32;                     // accumulator blocks per staging pass

    f32x16 acc[NI];
    // accumulators start from the bias (zeros without one): 4 columns per 16-byte read
    auto reset_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const float4 b4 = *reinterpret_cast<const float4 *>(sBias + j * 32 + 8 * g4 + 4 * frag_kg);
                acc[j][4 * g4 + 0] = b4.x; acc[j][4 * g4 + 1] = b4.y; acc[j][4 * g4 + 2] = b4.z; acc[j][4 * g4 + 3] = b4.w;
            }
    };
    // fp32 -> bf16 (nearest even) of one pass of JN blocks into the staging area
    auto stage_out = [&](int jc, auto relu_c) __attribute__((always_inline)) {
        constexpr bool RELU = decltype(relu_c)::value;
#pragma unroll
        for (int jj = 0; jj < JN; ++jj) {
            const int j = jc * JN + jj;
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int c = jj * 4 + g4;
                uint2 pk = make_uint2(pack_bf16x2(acc[j][4 * g4], acc[j][4 * g4 + 1]), pack_bf16x2(acc[j][4 * g4 + 2], acc[j][4 * g4 + 3]));
                if (RELU) {                         // max(0, .) on the bf16 pairs: as 16-bit integers, negative values are < 0
                    pk.x = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, pk.x), s16x2{0, 0}));
                    pk.y = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, pk.y), s16x2{0, 0}));
                }
                *reinterpret_cast<uint2 *>(stg + frag_row * EW + stg_chunk(frag_row, c) + 4 * (frag_kg ^ ((frag_row >> 3) & 1))) = pk;
            }
        }
    };

    // Operand fetch.  The filter is resident, so its fragments for the coming stage are requested BEFORE the
    // barrier that publishes the stage (HB k-steps of them: all four while that fits the register budget) and
    // arrive while the wave waits there; after the barrier only the activation fragments are fetched, all four
    // k-steps at once, and the MFMAs run as they arrive.
    constexpr int KS = BK / 16;
    constexpr int HB = NI <= 2 ? KS : KS / 2;       // k-steps of filter fragments held at a time
    bf16x8 bq[HB][NI];
    auto fetch_b = [&](int kt_of, int ks0) __attribute__((always_inline)) {
        const bf16_t *b_st = b_base + (size_t)kt_of * BN * BK;
#pragma unroll
        for (int h = 0; h < HB; ++h) {
            const int pos = (((ks0 + h) * 2 + frag_kg) ^ frag_swz) << 3;
#pragma unroll
            for (int j = 0; j < NI; ++j) bq[h][j] = *reinterpret_cast<const bf16x8 *>(b_st + j * 32 * BK + pos);
        }
    };

    // Stores of the common case (output pixel index == GEMM row, no mask): one buffer store per 8 staged rows;
    // rows past the end of this workgroup's range and columns past Co get an offset the resource rejects.
    const out_rsrc_t rs_out = make_out_rsrc(p.out, sp.out_bytes);
    const bool fast_store = p.linear_out && p.mask == nullptr;
    constexpr int RPI = 64 / CPR;                   // staged rows per store instruction
    const int st_r = lane / CPR, st_c = lane % CPR;
    const unsigned st_lane_off = (unsigned)((st_r * p.Co + n0 + st_c * 8) * 2);
    const bf16_t *st_src = stg + st_r * EW + stg_chunk(st_r, st_c);   // RPI is a multiple of CPR << LB: same chunk position for every k

    wait_vmcnt<0>();                                // this wave's share of the filter
    wg_barrier();                                   // filter and stage 0 complete
    reset_acc();
    int slot = 0, kt = 0, tile = 0;
    if (total > 0) fetch_b(0, 0);
    for (int g = 0; g < total; ++g) {
        const bf16_t *a_st = a_base + slot * STG_A;
        bf16x8 a[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) a[ks] = *reinterpret_cast<const bf16x8 *>(a_st + (((ks * 2 + frag_kg) ^ frag_swz) << 3));
#pragma unroll
        for (int h0 = 0; h0 < KS; h0 += HB) {
            if (h0 > 0) fetch_b(kt, h0);            // second half of the stage into the same registers
#pragma unroll
            for (int h = 0; h < HB; ++h)
#pragma unroll
                for (int j = 0; j < NI; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq[h][j], a[h0 + h], acc[j], 0, 0, 0);
        }
        // every activation fragment of this slot has been consumed by an MFMA, so its read has returned: the
        // slot can be handed back.  The filter fragments of the next stage are requested first.
        const int kt_next = kt + 1 == KT ? 0 : kt + 1;
        if (g + 1 < total) fetch_b(kt_next, 0);
        wg_barrier();
        slot = slot + 1 == NS ? 0 : slot + 1;
        kt = kt_next;
        if (kt != 0) continue;
        // ---- tile finished: ReLU, conversion, staging, mask, 16-byte stores ---------------------------------
        const int m0 = wg_lo + tile * BM + wave * 32;
        ++tile;
#pragma unroll
        for (int jc = 0; jc < (BN + 63) / 64; ++jc) {
            if (p.relu) stage_out(jc, std::true_type{});
            else stage_out(jc, std::false_type{});
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (fast_store) {
                const bool col_ok = n0 + jc * 64 + st_c * 8 < p.Co;
                const unsigned tile_off = (unsigned)m0 * (unsigned)(p.Co * 2) + (unsigned)(jc * 128);   // below 2^32: the output is below 2^31
                const int rows_left = wg_hi - m0;
#pragma unroll
                for (int k = 0; k < 32 / RPI; ++k) {
                    const uint4 v = swap_halves(*reinterpret_cast<const uint4 *>(st_src + k * RPI * EW), ((st_r + k * RPI) >> 3) & 1);
                    const bool ok = col_ok && st_r + k * RPI < rows_left;
                    if (sp.nt & 1) buffer_store16_nt(rs_out, ok ? st_lane_off + tile_off + (unsigned)(k * RPI * p.Co * 2) : OOB, v);
                    else buffer_store16(rs_out, ok ? st_lane_off + tile_off + (unsigned)(k * RPI * p.Co * 2) : OOB, v);
                }
            } else
#pragma unroll
            for (int k = 0; k < 32 * CPR / 64; ++k) {
                const int idx = k * 64 + lane;
                const int r = idx / CPR, c = idx % CPR;
                const int m = m0 + r, co = n0 + jc * 64 + c * 8;
                uint4 v = swap_halves(*reinterpret_cast<const uint4 *>(stg + r * EW + stg_chunk(r, c)), (r >> 3) & 1);
                if (m < wg_hi && co < p.Co) {
                    long long pix = m;
                    if (!p.linear_out) {
                        const unsigned b = (unsigned)m % (unsigned)p.Mw, t2 = (unsigned)m / (unsigned)p.Mw;
                        const unsigned a = t2 % (unsigned)p.Mh, n = t2 / (unsigned)p.Mh;
                        pix = ((long long)n * p.Ho + ((int)a * p.out_mul_h + p.out_off_h)) * p.Wo + ((int)b * p.out_mul_w + p.out_off_w);
                    }
                    const long long off = pix * p.Co + co;
                    if (p.mask != nullptr) {
                        const uint4 mk = *reinterpret_cast<const uint4 *>(p.mask + off);
                        v = make_uint4(mask_bf16x2(v.x, mk.x), mask_bf16x2(v.y, mk.y), mask_bf16x2(v.z, mk.z), mask_bf16x2(v.w, mk.w));
                    }
                    *reinterpret_cast<uint4 *>(p.out + off) = v;
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
        reset_acc();
    }
}

struct StreamConfig { int nc, ns, bn, lds; bool ok; };

// LDS bytes of a configuration: resident filter tile, ring, per-wave staging, tap table
long long stream_lds(int nc, int ns, int bn, int KT)
{
    const int ew = bn < 64 ? bn : 64;
    return (long long)bn * KT * BK * 2 + (long long)ns * 32 * nc * BK * 2 + (long long)nc * 32 * ew * 2 + (MAX_TAPS + 1) * 8 + bn * 4;
}

// The forms the kernel is built in, (compute waves, ring stages), in the order of preference measured on 1x1
// layers of 56x56 and 28x28 images: eight compute waves where the filter tile leaves room for their ring (the
// epilogue of a tile - conversion, staging, stores - is shared by more waves), else four with a deeper ring.
// MXC_STREAM_SHAPE=<compute waves>x<stages> (tuning sweeps only) picks one.
const int kForms[][2] = {{8, 3}, {4, 4}, {4, 3}, {4, 6}};

// Column tile: the smallest of 32 / 64 / 128 that holds min(Co, 128).
StreamConfig stream_config(const IgemmParams &p)
{
    const int Kd = p.TR * p.TS * p.Ci, KT = (Kd + BK - 1) / BK;
    const int bn = p.Co <= 32 ? 32 : p.Co <= 64 ? 64 : 128;
    int want_nc = 0, want_ns = 0;
    if (const char *f = getenv("MXC_STREAM_SHAPE")) {
        if (sscanf(f, "%dx%d", &want_nc, &want_ns) != 2) want_nc = want_ns = 0;
    }
    for (const auto &f : kForms) {
        if (want_nc && (f[0] != want_nc || f[1] != want_ns)) continue;
        const long long lds = stream_lds(f[0], f[1], bn, KT);
        if (lds <= 160 * 1024) return StreamConfig{f[0], f[1], bn, (int)lds, true};
    }
    return StreamConfig{0, 0, 0, 0, false};
}

template <int NC, int NL, int BN, int NS>
int launch_stream(StreamParams sp, int lds, hipStream_t st)
{
    static bool attr_set = false;      // raising the dynamic-LDS limit is idempotent; racing threads set the same value
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&stream_kernel<NC, NL, BN, NS>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                160 * 1024) != hipSuccess)
            return MXC_ERR_LAUNCH;
        attr_set = true;
    }
    IgemmParams &p = sp.g;
    constexpr int BM = 32 * NC;
    p.m_tiles = (int)(((long long)p.m_end - p.m_begin + BM - 1) / BM);
    p.n_tiles = (p.Co + BN - 1) / BN;
    // persistent grid: as many workgroups per CU as the LDS holds (at most 12 waves), shared by the column tiles
    int per_cu = (160 * 1024) / lds;
    if (per_cu > 12 / (NC + NL)) per_cu = 12 / (NC + NL);
    int n_wg_m = (256 * per_cu) / p.n_tiles;
    if (n_wg_m < 1) n_wg_m = 1;
    if (n_wg_m > p.m_tiles) n_wg_m = p.m_tiles;
    const long long rows = (long long)p.m_end - p.m_begin;
    sp.rows_per_wg = (int)(((rows + n_wg_m - 1) / n_wg_m + 31) / 32 * 32);
    n_wg_m = (int)((rows + sp.rows_per_wg - 1) / sp.rows_per_wg);
    sp.n_wg_m = n_wg_m;
    sp.units = n_wg_m * p.n_tiles;
    sp.per_xcd = ((sp.units + 7) / 8 + p.n_tiles - 1) / p.n_tiles * p.n_tiles;
    // Cache policy, measured on 1x1 layers of 56x56 images: results of a large layer leave as non-temporal stores
    // (the next reader finds them in HBM whatever the policy, and the caches keep serving this kernel's reads);
    // activations that no second workgroup and no second tap will ask for arrive as non-temporal loads.
    // MXC_STREAM_NT=<bits> (tuning sweeps only) overrides.
    const long long in_bytes = (long long)p.N * p.Hi * p.Wi * p.pix * 2, out_bytes = (long long)p.N * p.Ho * p.Wo * p.Co * 2;
    sp.nt = (out_bytes >= (32ll << 20) ? 1 : 0) | ((in_bytes >= (64ll << 20) && p.n_tiles == 1 && p.TR * p.TS == 1) ? 2 : 0);
    if (const char *f = getenv("MXC_STREAM_NT")) sp.nt = atoi(f);
    sp.out_bytes = (unsigned)((long long)p.N * p.Ho * p.Wo * p.Co * 2);
    sp.d_n = BM / (p.Mh * p.Mw);
    sp.d_a = BM % (p.Mh * p.Mw) / p.Mw;
    sp.d_b = BM % p.Mw;
    hipLaunchKernelGGL((stream_kernel<NC, NL, BN, NS>), dim3((unsigned)(8 * sp.per_xcd)), dim3(64 * (NC + NL)), (size_t)lds, st, sp);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

template <int NC, int NL, int NS>
int launch_stream_bn(const StreamParams &sp, const StreamConfig &c, hipStream_t st)
{
    if (c.bn == 32) return launch_stream<NC, NL, 32, NS>(sp, c.lds, st);
    if (c.bn == 64) return launch_stream<NC, NL, 64, NS>(sp, c.lds, st);
    return launch_stream<NC, NL, 128, NS>(sp, c.lds, st);
}

}  // namespace

bool stream_applicable(const IgemmParams &p)
{
    if (p.splits > 1 || p.partial != nullptr) return false;
    const int Kd = p.TR * p.TS * p.Ci;
    if ((long long)p.N * p.Mh * p.Mw >= 0x7FFF0000ll) return false;          // row indices plus a tile stay in 31 bits
    if ((long long)p.N * p.Ho * p.Wo * p.Co * 2 >= 0x7FFF0000ll) return false;   // 32-bit byte offsets into the output
    if (Kd % 8 != 0 || p.Ci % 8 != 0 || (p.Co & 7) != 0) return false;      // 16-byte chunks within a tap's run; 16-byte stores
    if (p.TR * p.TS > MAX_TAPS) return false;
    return stream_config(p).ok;
}

int stream_launch(const IgemmParams &p, hipStream_t st)
{
    const StreamConfig c = stream_config(p);
    if (!c.ok) return MXC_ERR_UNSUPPORTED;
    StreamParams sp{};
    sp.g = p;
    IgemmParams &q = sp.g;
    const long long M = (long long)p.N * p.Mh * p.Mw;
    if (M <= 0) return MXC_OK;
    q.M = (int)M;
    q.m_begin = 0;
    q.m_end = (int)M;
    q.in_bytes = (unsigned)((long long)p.N * p.Hi * p.Wi * p.pix * 2);
    q.wm_bytes = (unsigned)((long long)p.Co * p.TR * p.TS * p.Ci * 2);
    q.tap_inner = 0;
    q.linear_out = (p.out_mul_h == 1 && p.out_mul_w == 1 && p.out_off_h == 0 && p.out_off_w == 0 && p.Mh == p.Ho && p.Mw == p.Wo) ? 1 : 0;
    const int Kd = p.TR * p.TS * p.Ci;
    sp.KT = (Kd + BK - 1) / BK;
    sp.b_bytes = c.bn * sp.KT * BK * 2;
    if (c.nc == 8) return launch_stream_bn<8, 4, 3>(sp, c, st);
    if (c.ns == 6) return launch_stream_bn<4, 2, 6>(sp, c, st);
    if (c.ns == 4) return launch_stream_bn<4, 2, 4>(sp, c, st);
    return launch_stream_bn<4, 2, 3>(sp, c, st);
}

}  // namespace mxc
