// Implicit GEMM from an LDS-resident input window and an LDS-resident filter: multi-tap stride-1 layers with at
// most 64 input channels and few output columns (3x3 layers of 64 channels, first layers after re-packing).
//
// Same GEMM as igemm.hip,  Out[m][co] = sum_{t,ci} In[pixel(m) + tap(t)][ci] * Wm[co][t*Ci + ci].  The tiled and the
// streaming kernel fetch, for every tap, the rows of their activation tile again: a layer with T taps pulls its
// input through the L2 T times.  Here an output tile is a 2-D PATCH of TH x TW pixels of one image (TW a multiple
// of 32, TH*TW = 256).  The (TH+R-1) x (TW+S-1) input pixels the patch touches - the window - are loaded ONCE into
// LDS, with the zero padding applied by the load (out-of-image pixels get an offset the buffer resource rejects),
// and every tap reads its operand fragments from the window at a shifted pixel index.  The filter tile of the
// workgroup's column tile stays in LDS for the kernel's lifetime, so between the barrier that hands a window over
// and the barrier that ends the patch a compute wave runs all its T * Ci/16 * BN/32 MFMAs without meeting anyone.
//   * workgroups are persistent and walk a contiguous range of patches; two window buffers alternate: the next
//     patch's window is loaded while this one is multiplied;
//   * waves are specialised as in the streaming kernel: 4 loader waves issue the asynchronous global->LDS loads,
//     8 compute waves (32 patch pixels each, all BN columns) read fragments, run the MFMAs
//     (v_mfma_f32_32x32x16_bf16, product formed transposed so a lane holds four neighbouring output columns) and
//     store; the finished window buffer serves as the staging area of the 16-byte result stores;
//   * fragments of tap t+1 are requested before the MFMAs of tap t are issued (two register sets).
// Window pixel P keeps its 8 16-byte channel chunks at positions c ^ ((P/2) % 8) of a 128-byte row.  A wave's 32
// rows are 32 consecutive window pixels (TW is a multiple of 32), whatever the tap: measured, fragment reads of 32
// consecutive pixels are free of bank conflicts from any starting pixel, reads of two runs of 16 are not.
#include <type_traits>

#include "mxc_internal.h"

namespace mxc {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x2 __attribute__((ext_vector_type(2)));

constexpr unsigned OOB = 0x80000000u;   // a buffer offset no operand reaches: the load returns zeros
constexpr int NC = 8;                   // compute waves: 256 patch pixels
constexpr int NL = 4;                   // loader waves
constexpr int NW = NC + NL;

template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
__device__ __forceinline__ void wg_barrier()
{
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
}

struct WindowParams {
    IgemmParams g;
    int TH, TW;          // output patch (TH*TW <= 256, TW % 32 == 0)
    int WH, WW;          // window = patch + taps - 1
    int PY, PX;          // patches per image
    int NP;              // patches in all = N*PY*PX
    int tiles_per_wg;    // workgroup w of a column tile owns patches [w*tiles_per_wg, (w+1)*tiles_per_wg)
    int units, per_xcd;  // workgroups in all, and per XCD (a multiple of n_tiles)
    int LWT;             // wave-wide loads per window = ceil(WH*WW / 8)
    int win_bytes;       // bytes of one window buffer (>= the staging area)
    int b_bytes;         // bytes of the resident filter tile: T * BN * 128
    int oy, ox;          // window origin relative to the patch origin, input coordinates
    unsigned ww_magic;   // ceil(2^22 / WW): exact quotients for dividends < 2^14
    int dq, dr;          // 32 = dq*WW + dr: one loader wave's next load lies 32 window pixels further on
    unsigned out_bytes;
    int nt;              // results leave as non-temporal stores
};

// Column tile BN = 32*NI; KSN = Ci/16 k-steps per tap.  Dynamic LDS: [filter T x BN x 64][window 0][window 1][bias BN][tap shifts].
template <int NI, int KSN>
__global__ __launch_bounds__(64 * NW) void window_kernel(const WindowParams wp)
{
    const IgemmParams &p = wp.g;
    constexpr int BN = 32 * NI;

    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    bf16_t *sB = reinterpret_cast<bf16_t *>(smem);
    bf16_t *win0 = reinterpret_cast<bf16_t *>(smem + wp.b_bytes);
    float *sBias = reinterpret_cast<float *>(smem + wp.b_bytes + 2 * (size_t)wp.win_bytes);
    int *tap_shift = reinterpret_cast<int *>(sBias + BN);
    const int win_elems = wp.win_bytes / 2;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave >= NC;

    const int unit = (blockIdx.x & 7) * wp.per_xcd + (blockIdx.x >> 3);
    if (unit >= wp.units) return;
    const int n_tile = unit % p.n_tiles, wg = unit / p.n_tiles;
    const int n0 = n_tile * BN;
    const int q_lo = wg * wp.tiles_per_wg;
    const int q_hi = min(wp.NP, q_lo + wp.tiles_per_wg);
    const int my_tiles = q_hi > q_lo ? q_hi - q_lo : 0;
    const int T = p.TR * p.TS;
    const int Kd = T * p.Ci;

    // tap t reads window pixel (ty + wy_t, tx + wx_t): shift = wy_t*WW + wx_t
    for (int t = tid; t < T; t += 64 * NW) {
        const int dh = p.tap_row_inner ? t % p.TR : t / p.TS, dv = p.tap_row_inner ? t / p.TR : t % p.TS;
        const int wy = p.tstep_h > 0 ? dh : p.TR - 1 - dh, wx = p.tstep_w > 0 ? dv : p.TS - 1 - dv;
        tap_shift[t] = wy * wp.WW + wx;
    }
    for (int c = tid; c < BN; c += 64 * NW) sBias[c] = (p.bias != nullptr && n0 + c < p.Co) ? p.bias[n0 + c] : 0.f;

    const buf_rsrc_t rs_in = make_buf_rsrc(p.in, p.in_bytes);
    const buf_rsrc_t rs_wm = make_buf_rsrc(p.wm, p.wm_bytes);

    // ---- resident filter: every wave fetches its share once.  Tap t is a [BN rows][64 channels] slab; row r keeps
    // 16-byte chunk c at position c ^ ((r/2) % 8); channels past Ci and rows past Co are zeros.
    {
        constexpr int per_tap = BN / 8;             // wave-wide loads per tap (8 rows each)
        for (int idx = wave; idx < T * per_tap; idx += NW) {
            const int t = idx / per_tap, i = idx % per_tap;
            const int r = 8 * i + (lane >> 3);
            const int kc = ((lane & 7) ^ ((r >> 1) & 7)) << 3;
            const unsigned off = (n0 + r < p.Co && kc < p.Ci) ? (unsigned)(n0 + r) * (unsigned)(Kd * 2) + (unsigned)((t * p.Ci + kc) * 2) : OOB;
            lds_dma16(rs_wm, off, sB + (size_t)t * BN * 64 + i * 8 * 64);
        }
    }

    __syncthreads();        // tap shifts and bias visible (the filter loads stay in flight)

    // Patch walk: (image, patch row, patch column) of the workgroup's first patch by division, then by counting.
    struct PatchPos { int n, py, px; };
    auto first_patch = [&]() __attribute__((always_inline)) {
        const int per_img = wp.PY * wp.PX;
        PatchPos pp;
        pp.n = q_lo / per_img;
        const int r = q_lo - pp.n * per_img;
        pp.py = r / wp.PX;
        pp.px = r - pp.py * wp.PX;
        return pp;
    };
    auto next_patch = [&](PatchPos &pp) __attribute__((always_inline)) {
        if (++pp.px == wp.PX) {
            pp.px = 0;
            if (++pp.py == wp.PY) {
                pp.py = 0;
                ++pp.n;
            }
        }
    };

    if (loader) {
        // =============================== loader waves ===================================================
        // This wave's k-th load of a window covers pixels 8*(l + NL*k) .. +7; lane -> pixel 8*(l + NL*k) + lane/8,
        // chunk position lane%8.  From one load to the next the pixel index grows by 32, so the swizzle term
        // (P/2) % 8 - and with it the logical chunk a lane fetches - never changes, and the pixel's window
        // coordinates advance by (dq, dr) with one wrap.
        const int l = wave - NC;
        const int P_first = 8 * l + (lane >> 3);
        const int wy_first = (int)(((unsigned)P_first * wp.ww_magic) >> 22), wx_first = P_first - wy_first * wp.WW;
        const int w_kc = ((lane & 7) ^ ((P_first >> 1) & 7)) << 3;   // first channel of this lane's chunk
        const int loads_per_window = (wp.LWT - l + NL - 1) / NL;     // of this wave
        const unsigned pix_bytes = (unsigned)(p.Ci * 2), row_bytes = (unsigned)(p.Wi * p.Ci * 2);
        const bool chunk_ok = w_kc < p.Ci;
        PatchPos pos = first_patch();
        // all loads of the window of patch `pos` into buffer `buf`
        auto request_window = [&](int buf) __attribute__((always_inline)) {
            const int yb = pos.py * wp.TH + wp.oy, xb = pos.px * wp.TW + wp.ox;   // input coordinates of window pixel (0, 0)
            // byte offset of (image, yb, xb, this lane's chunk): wraps below zero in the padding, exact where the pixel is valid
            const unsigned base = (unsigned)(((pos.n * p.Hi + yb) * p.Wi + xb) * p.Ci * 2) + (unsigned)(w_kc * 2);
            bf16_t *dst = win0 + buf * win_elems + l * 512;
            int wy = wy_first, wx = wx_first;
            for (int k = 0; k < loads_per_window; ++k) {
                const int y = yb + wy, x = xb + wx;
                const bool ok = chunk_ok && (unsigned)y < (unsigned)p.Hi && (unsigned)x < (unsigned)p.Wi;
                lds_dma16(rs_in, ok ? base + (unsigned)wy * row_bytes + (unsigned)wx * pix_bytes : OOB, dst);
                dst += NL * 512;
                wy += wp.dq;
                wx += wp.dr;
                const bool wrap = wx >= wp.WW;
                wx -= wrap ? wp.WW : 0;
                wy += wrap ? 1 : 0;
            }
        };
        if (my_tiles > 0) request_window(0);
        for (int k = 0; k < my_tiles; ++k) {
            wait_vmcnt<0>();                        // this wave's share of window k (and, the first time, of the filter)
            wg_barrier();                           // A(k): window k is whole; every compute wave is done with patch k-1, stores included
            if (k + 1 < my_tiles) {
                next_patch(pos);
                request_window((k + 1) & 1);        // the buffer patch k-1 used, free since A(k)
            }
            wg_barrier();                           // B(k)
        }
        wait_vmcnt<0>();
        return;
    }

    // ================================= compute waves =======================================================
    const int frag_row = lane & 31, frag_kg = lane >> 5;
    const int frag_swz = (frag_row >> 1) & 7;
    const bf16_t *b_base = sB + frag_row * 64;
    constexpr int EW = NI * 32;                     // staging width (columns)
    static_assert(NI == 1 || NI == 2, "one staging pass");
    constexpr int CPR = EW / 8;                     // 16-byte chunks per staged row
    constexpr int LBS = EW == 64 ? 0 : 1;           // log2 of the rows that share one 128-byte line of banks
    constexpr int RPI = 64 / CPR;                   // staged rows per store instruction
    auto stg_chunk = [](int r, int c) __attribute__((always_inline)) { return (c ^ ((r >> LBS) & (CPR - 1))) << 3; };

    // window pixel of this lane's row (patch-relative, tap 0): TW is a multiple of 32, so a wave's 32 rows are one run
    const int row0 = wave * 32;
    // (rows past a short patch read pixels 0..31: their results are not stored)
    const int pbase = (row0 < wp.TH * wp.TW ? (row0 / wp.TW) * wp.WW + row0 % wp.TW : 0) + frag_row;
    // result stores: lane -> staged row st_r + k*RPI, chunk st_c; patch-relative byte offset and (ty, tx)
    const int st_r = lane / CPR, st_c = lane % CPR;
    unsigned st_off[32 / RPI];
    int st_yx[32 / RPI];
#pragma unroll
    for (int k = 0; k < 32 / RPI; ++k) {
        const int r = row0 + st_r + k * RPI;
        const int ty = r / wp.TW, tx = r % wp.TW;
        st_off[k] = (unsigned)(((ty * p.Wo + tx) * p.Co + n0 + st_c * 8) * 2);
        st_yx[k] = r < wp.TH * wp.TW ? (ty | (tx << 16)) : 0x7FFF;
    }
    const bool st_col_ok = n0 + st_c * 8 < p.Co;
    const out_rsrc_t rs_out = make_out_rsrc(p.out, wp.out_bytes);

    f32x16 acc[NI];
    auto reset_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const float4 b4 = *reinterpret_cast<const float4 *>(sBias + j * 32 + 8 * g4 + 4 * frag_kg);
                acc[j][4 * g4 + 0] = b4.x; acc[j][4 * g4 + 1] = b4.y; acc[j][4 * g4 + 2] = b4.z; acc[j][4 * g4 + 3] = b4.w;
            }
    };
    struct Frags { bf16x8 a[KSN]; bf16x8 b[KSN][NI]; };
    auto fetch = [&](Frags &f, int t, const bf16_t *w_st) __attribute__((always_inline)) {
        const int P = pbase + tap_shift[t];
        const bf16_t *row = w_st + P * 64;
        const int swz = (P >> 1) & 7;
        const bf16_t *b_t = b_base + (size_t)t * BN * 64;
#pragma unroll
        for (int ks = 0; ks < KSN; ++ks) {
            f.a[ks] = *reinterpret_cast<const bf16x8 *>(row + (((ks * 2 + frag_kg) ^ swz) << 3));
#pragma unroll
            for (int j = 0; j < NI; ++j) f.b[ks][j] = *reinterpret_cast<const bf16x8 *>(b_t + j * 32 * 64 + (((ks * 2 + frag_kg) ^ frag_swz) << 3));
        }
        __builtin_amdgcn_sched_barrier(0);          // the reads stay ahead of the MFMAs that follow in program order
    };
    auto mma = [&](const Frags &f) __attribute__((always_inline)) {
#pragma unroll
        for (int ks = 0; ks < KSN; ++ks)
#pragma unroll
            for (int j = 0; j < NI; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[ks][j], f.a[ks], acc[j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
    };

    wait_vmcnt<0>();                                // this wave's share of the filter
    PatchPos pos = first_patch();
    for (int k = 0; k < my_tiles; ++k) {
        wg_barrier();                               // A(k): window k and (the first time) the filter are whole
        if (k == 0) reset_acc();                    // the bias vector became visible with the barrier
        const bf16_t *w_st = win0 + (k & 1) * win_elems;
        Frags f0, f1;
        fetch(f0, 0, w_st);
        int t = 0;
        for (; t + 2 <= T; t += 2) {
            fetch(f1, t + 1, w_st);
            mma(f0);
            if (t + 2 < T) fetch(f0, t + 2, w_st);
            mma(f1);
        }
        if (t < T) mma(f0);
        wg_barrier();                               // B(k): every wave is done reading window k, which becomes the staging area
        {
            const int n = pos.n, y0 = pos.py * wp.TH, x0 = pos.px * wp.TW;
            next_patch(pos);
            const int th = min(wp.TH, p.Mh - y0), tw = min(wp.TW, p.Mw - x0);
            const int lim = (th - 1) | ((tw - 1) << 16);
            const unsigned tile_off = (unsigned)(((n * p.Ho + y0) * p.Wo + x0) * p.Co * 2);   // below 2^31: the output is
            bf16_t *stg = win0 + (k & 1) * win_elems + wave * 32 * EW;
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int c = j * 4 + g4;
                    uint2 pk = make_uint2(pack_bf16x2(acc[j][4 * g4], acc[j][4 * g4 + 1]), pack_bf16x2(acc[j][4 * g4 + 2], acc[j][4 * g4 + 3]));
                    if (p.relu) {                   // max(0, .) on the bf16 pairs: as 16-bit integers, negative values are < 0
                        pk.x = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, pk.x), s16x2{0, 0}));
                        pk.y = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, pk.y), s16x2{0, 0}));
                    }
                    *reinterpret_cast<uint2 *>(stg + frag_row * EW + stg_chunk(frag_row, c) + 4 * (frag_kg ^ ((frag_row >> 3) & 1))) = pk;
                }
            reset_acc();
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int kk = 0; kk < 32 / RPI; ++kk) {
                const int r = st_r + kk * RPI;
                uint4 v = *reinterpret_cast<const uint4 *>(stg + r * EW + stg_chunk(r, st_c));
                if ((r >> 3) & 1) v = make_uint4(v.z, v.w, v.x, v.y);
                // inside the patch's valid part: ty <= th-1 and tx <= tw-1, tested on both halves at once
                const s16x2 d = __builtin_bit_cast(s16x2, lim) - __builtin_bit_cast(s16x2, st_yx[kk]);
                const bool ok = st_col_ok && (__builtin_bit_cast(int, d) & (int)0x80008000) == 0;
                const unsigned off = ok ? tile_off + st_off[kk] : OOB;
                if (wp.nt) buffer_store16_nt(rs_out, off, v);
                else buffer_store16(rs_out, off, v);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
}

struct WindowConfig { int bn, th, tw, lds, win_bytes; bool ok; };

// bytes of one window buffer: the window in whole wave-wide loads, at least the store staging area (32 rows x bn columns
// per compute wave)
int window_bytes(int th, int tw, int TR, int TS, int bn)
{
    const int px = (th + TR - 1) * (tw + TS - 1);
    const int b = (px + 7) / 8 * 1024, staging = NC * 32 * bn * 2;
    return b < staging ? staging : b;
}

// Patch shape: TW in {32, 64, 128, 256}, TH = 256 / TW (at most the image height); the one that wastes the fewest rows
// of the 256-row tiles over an image, ties to the smaller window.  MXC_WINDOW_PATCH=<th>x<tw> (tuning sweeps only).
WindowConfig window_config(const IgemmParams &p)
{
    const int T = p.TR * p.TS;
    const int bn = p.Co <= 32 ? 32 : 64;
    WindowConfig best{bn, 0, 0, 0, 0, false};
    int want_th = 0, want_tw = 0;
    if (const char *f = getenv("MXC_WINDOW_PATCH")) {
        if (sscanf(f, "%dx%d", &want_th, &want_tw) != 2 || want_th < 1 || want_tw < 32 || want_tw % 32 || want_th * want_tw > 256) want_th = want_tw = 0;
    }
    double best_score = 0;
    for (int tw = 32; tw <= 256; tw *= 2) {
        int th = 256 / tw;
        if (th > p.Mh) th = p.Mh;
        if (want_th) {
            if (tw != want_tw) continue;
            th = want_th;
        }
        const int wb = window_bytes(th, tw, p.TR, p.TS, bn);
        const long long lds = (long long)T * bn * 128 + 2ll * wb + bn * 4 + (MAX_TAPS + 1) * 4;
        if (lds > 160 * 1024) continue;
        const long long tiles = (long long)((p.Mh + th - 1) / th) * ((p.Mw + tw - 1) / tw);
        const double eff = (double)p.Mh * p.Mw / (double)(tiles * 256);
        const double score = eff - 1e-3 * (double)wb / (160.0 * 1024);
        if (score > best_score) {
            best_score = score;
            best = WindowConfig{bn, th, tw, (int)lds, wb, true};
        }
    }
    return best;
}

template <int NI, int KSN>
int launch_window(WindowParams &wp, int lds, hipStream_t st)
{
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&window_kernel<NI, KSN>), hipFuncAttributeMaxDynamicSharedMemorySize,
                                160 * 1024) != hipSuccess)
            return MXC_ERR_LAUNCH;
        attr_set = true;
    }
    hipLaunchKernelGGL((window_kernel<NI, KSN>), dim3((unsigned)(8 * wp.per_xcd)), dim3(64 * NW), (size_t)lds, st, wp);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

template <int NI>
int launch_window_ks(WindowParams &wp, int lds, hipStream_t st)
{
    switch (wp.g.Ci / 16) {
    case 1: return launch_window<NI, 1>(wp, lds, st);
    case 2: return launch_window<NI, 2>(wp, lds, st);
    case 3: return launch_window<NI, 3>(wp, lds, st);
    default: return launch_window<NI, 4>(wp, lds, st);
    }
}

}  // namespace

bool window_applicable(const IgemmParams &p)
{
    if (p.splits > 1 || p.partial != nullptr || p.mask != nullptr || p.f32_out) return false;
    const int T = p.TR * p.TS;
    if (T < 2 || T > MAX_TAPS) return false;
    if (p.in_mul_h != 1 || p.in_mul_w != 1 || (p.tstep_h != 1 && p.tstep_h != -1) || (p.tstep_w != 1 && p.tstep_w != -1)) return false;
    if (p.pix != p.Ci || p.Ci % 16 != 0 || p.Ci > 64 || (p.Co & 7) != 0) return false;
    if (!(p.out_mul_h == 1 && p.out_mul_w == 1 && p.out_off_h == 0 && p.out_off_w == 0 && p.Mh == p.Ho && p.Mw == p.Wo)) return false;
    if ((long long)p.N * p.Hi * p.Wi * p.Ci * 2 >= 0x7FFF0000ll) return false;      // 32-bit byte offsets into the input
    if ((long long)p.N * p.Ho * p.Wo * p.Co * 2 >= 0x7FFF0000ll) return false;      // ... and the output
    if (p.Mh > 0x7FFF || p.Mw > 0x7FFF) return false;
    return window_config(p).ok;
}

int window_launch(const IgemmParams &p, hipStream_t st)
{
    const WindowConfig c = window_config(p);
    if (!c.ok) return MXC_ERR_UNSUPPORTED;
    if ((long long)p.N * p.Mh * p.Mw <= 0) return MXC_OK;
    WindowParams wp{};
    wp.g = p;
    IgemmParams &q = wp.g;
    const int T = p.TR * p.TS;
    q.in_bytes = (unsigned)((long long)p.N * p.Hi * p.Wi * p.Ci * 2);
    q.wm_bytes = (unsigned)((long long)p.Co * T * p.Ci * 2);
    q.n_tiles = (p.Co + c.bn - 1) / c.bn;
    wp.TH = c.th;
    wp.TW = c.tw;
    wp.WH = c.th + p.TR - 1;
    wp.WW = c.tw + p.TS - 1;
    wp.PY = (p.Mh + c.th - 1) / c.th;
    wp.PX = (p.Mw + c.tw - 1) / c.tw;
    const long long NP = (long long)p.N * wp.PY * wp.PX;
    if (NP > 0x3FFFFFFFll) return MXC_ERR_SHAPE;
    wp.NP = (int)NP;
    // persistent grid: one workgroup per CU, shared by the column tiles; every workgroup the same number of patches
    int n_wg = 256 / q.n_tiles;
    if (n_wg < 1) n_wg = 1;
    if (n_wg > wp.NP) n_wg = wp.NP;
    wp.tiles_per_wg = (wp.NP + n_wg - 1) / n_wg;
    n_wg = (wp.NP + wp.tiles_per_wg - 1) / wp.tiles_per_wg;
    wp.units = n_wg * q.n_tiles;
    wp.per_xcd = ((wp.units + 7) / 8 + q.n_tiles - 1) / q.n_tiles * q.n_tiles;
    wp.LWT = (wp.WH * wp.WW + 7) / 8;
    wp.win_bytes = c.win_bytes;
    wp.b_bytes = T * c.bn * 128;
    wp.oy = p.in_off_h + (p.tstep_h < 0 ? -(p.TR - 1) : 0);
    wp.ox = p.in_off_w + (p.tstep_w < 0 ? -(p.TS - 1) : 0);
    wp.ww_magic = (unsigned)(((1u << 22) + wp.WW - 1) / wp.WW);
    wp.dq = 32 / wp.WW;
    wp.dr = 32 % wp.WW;
    wp.out_bytes = (unsigned)((long long)p.N * p.Ho * p.Wo * p.Co * 2);
    wp.nt = (long long)wp.out_bytes >= (32ll << 20) ? 1 : 0;
    if (c.bn == 32) return launch_window_ks<1>(wp, c.lds, st);
    return launch_window_ks<2>(wp, c.lds, st);
}

}  // namespace mxc
