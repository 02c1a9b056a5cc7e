// Internal declarations shared by the library's translation units (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/mxc.h"

namespace mxc {

typedef uint16_t bf16_t;  // raw bf16 bit pattern

// One convolution problem in the library's working layout: activations NHWC,
// filters KRSC.  P and Q are derived by the ABI layer.
struct ConvShape {
    int N, C, H, W, K, R, S, stride, pad, P, Q;
};

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// Round-to-nearest-even; inputs are finite in this library's use.
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// two values at once (v_cvt_pk_bf16_f32): `lo` in bits 0..15; the same rounding as f32_to_bf16 for finite inputs
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ float load_f32(const float *p) { return *p; }
__device__ __forceinline__ float load_f32(const bf16_t *p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void store_f32(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_f32(bf16_t *p, float v) { *p = f32_to_bf16(v); }

// What the kernel that produces a result applies to it before the store (the grouped forms of the
// convolution: see mxc_conv2d_fwd_bias_act / mxc_conv2d_bwd_data_relu).  Default: nothing.
struct PostOp {
    const float *bias = nullptr;   // forward: + bias[k], one fp32 value per output channel
    int relu = 0;                  // forward: max(0, .) after the bias
    const void *mask = nullptr;    // backward-data: result is 0 where mask <= 0; same shape, type and layout as dx
};

// keeps the halves of v (two bf16) whose mask half is > 0
__device__ __forceinline__ uint32_t mask_bf16x2(uint32_t v, uint32_t m)
{
    const uint32_t lo = (int16_t)(m & 0xFFFFu) > 0 ? 0x0000FFFFu : 0u;
    const uint32_t hi = (int16_t)(m >> 16) > 0 ? 0xFFFF0000u : 0u;
    return v & (lo | hi);
}
__device__ __forceinline__ bool mask_keeps(const float *m) { return *m > 0.f; }
__device__ __forceinline__ bool mask_keeps(const bf16_t *m) { return (int16_t)*m > 0; }

// ---- asynchronous global -> LDS transfers (the MFMA kernels' operand path) ---------------------------
// A wave-wide 16-byte-per-lane buffer load whose data goes straight to LDS: lane l's 16 bytes land at
// lds_base + 16*l, where lds_base is wave-uniform.  Lanes whose byte offset lies outside the buffer deposit
// zeros (how padding, ragged edges and reduction tails are filled).
//
// Written as inline assembly on purpose.  Issued through the compiler's builtin, the transfer is known to the
// compiler as a write to LDS, and it then guards LDS reads that it cannot prove disjoint (every read made
// with a transposing-read builtin, every read after a control-flow join, everything once more than eight LDS
// objects are in play) with a wait for ALL outstanding transfers, which empties a ring of stages at every
// stage.  This way the compiler sees no LDS write at all; the kernels order the transfers against their LDS
// reads themselves (s_waitcnt vmcnt(N) + barrier before a stage is read).  M0 holds the LDS base for the
// instruction; nothing else in these kernels uses M0.
typedef int buf_rsrc_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ buf_rsrc_t make_buf_rsrc(const void *base, unsigned bytes)
{
    const uint64_t a = (uint64_t)base;
    buf_rsrc_t r;
    r.x = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    r.y = __builtin_amdgcn_readfirstlane((int)((uint32_t)(a >> 32) & 0xFFFFu));   // stride 0: raw buffer
    r.z = __builtin_amdgcn_readfirstlane((int)bytes);                              // out-of-range above this
    r.w = 0x00020000;
    return r;
}
__device__ __forceinline__ void lds_dma16(buf_rsrc_t rsrc, unsigned byte_off, const void *lds_base_uniform)
{
    typedef __attribute__((address_space(3))) const void *lds_cvptr;
    const unsigned lds_addr = (unsigned)(uintptr_t)(lds_cvptr)lds_base_uniform;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(byte_off), "s"(rsrc)
                 : "memory");
}

// lds_dma16 marked non-temporal: a streaming read that the caches need not keep
__device__ __forceinline__ void lds_dma16_nt(buf_rsrc_t rsrc, unsigned byte_off, const void *lds_base_uniform)
{
    typedef __attribute__((address_space(3))) const void *lds_cvptr;
    const unsigned lds_addr = (unsigned)(uintptr_t)(lds_cvptr)lds_base_uniform;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen nt lds"
                 :
                 : "s"(lds_addr), "v"(byte_off), "s"(rsrc)
                 : "memory");
}
// 16-byte store through a buffer resource: a lane whose byte_off lies beyond the resource's size writes nothing,
// which takes the place of a bounds branch.  These are compiler builtins, not inline assembly, so that the compiler
// itself keeps the wait states between a store wider than 8 bytes and the next write of its data registers.
typedef __amdgpu_buffer_rsrc_t out_rsrc_t;
__device__ __forceinline__ out_rsrc_t make_out_rsrc(void *base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, (int)bytes, 0x00020000);     // stride 0: raw buffer
}
__device__ __forceinline__ void buffer_store16(out_rsrc_t rsrc, unsigned byte_off, uint4 v)
{
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    __builtin_amdgcn_raw_buffer_store_b128(u32x4{v.x, v.y, v.z, v.w}, rsrc, (int)byte_off, 0, 0);
}
__device__ __forceinline__ void buffer_store16_nt(out_rsrc_t rsrc, unsigned byte_off, uint4 v)
{
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    __builtin_amdgcn_raw_buffer_store_b128(u32x4{v.x, v.y, v.z, v.w}, rsrc, (int)byte_off, 0, 2);   // 2: non-temporal
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline size_t elem_size(int dtype) { return dtype == MXC_BF16 ? 2 : 4; }

// ---- layout.hip ------------------------------------------------------------
// Batched 2-D transpose: src[b][rows][cols] -> dst[b][cols][rows], element size 2 or 4 bytes.
int launch_transpose(const void *src, void *dst, int batch, int rows, int cols, int elem_bytes,
                     hipStream_t stream);
// whether launch_transpose can run this problem (its grid holds batch x ceil(rows/64) x ceil(cols/64) workgroups)
bool transpose_launchable(long long batch, long long rows, long long cols);
int launch_copy(const void *src, void *dst, size_t bytes, hipStream_t stream);

// ---- probe.hip: matrix-pipe ceiling measurement -------------------------------------
// launches the register-resident MFMA loop; *flops = floating-point operations the launch performs
int probe_mfma(int workgroups, int iters, float *out, double *flops, hipStream_t st);

// ---- update.hip: SGD with momentum and weight decay on fp32 master weights -------------
int sgd_update(size_t n, float *w, const float *g, float *v, void *w_copy, float lr, float momentum, float wd, hipStream_t st);

// ---- softmax.hip: softmax output layer --------------------------------------------------
int softmax_fwd(int N, int K, int dtype, const void *z, void *p, hipStream_t st);
int softmax_xent_bwd(int N, int K, int dtype, const void *p, const int *labels, void *dz, float scale, hipStream_t st);

// ---- bias.hip: bias gradient ------------------------------------------------------------
int bias_grad_parts(long long N, int K, long long PQ, int layout);      // partial vectors of K floats the call needs as scratch
int bias_grad(long long N, int K, long long PQ, int dtype, int layout, const void *dy, float *db, float *partial, hipStream_t st);

// ---- direct.hip: one-thread-per-output kernels, any shape, NHWC/KRSC --------
int direct_fwd(const ConvShape &s, int dtype, const void *x, const void *w, void *y, hipStream_t st, const PostOp &post = PostOp());
int direct_bwd_data(const ConvShape &s, int dtype, const void *dy, const void *w, void *dx, hipStream_t st,
                    const PostOp &post = PostOp());
// partial: fp32 scratch of direct_bwd_weight_splits(s) * K*R*S*C floats
int direct_bwd_weight_splits(const ConvShape &s);
// dw: fp32, or bf16 (the fp32 sum rounded once) when dw_bf16
int direct_bwd_weight(const ConvShape &s, int dtype, const void *x, const void *dy, void *dw, bool dw_bf16,
                      float *partial, int splits, hipStream_t st);

// ---- igemm.hip: bf16 MFMA implicit GEMM (NHWC/KRSC) ---------------------------
bool igemm_fwd_supported(const ConvShape &s);
// split_ws: scratch of igemm_fwd_split_bytes(s) bytes for a split reduction (may be null: never split)
size_t igemm_fwd_split_bytes(const ConvShape &s);
int igemm_fwd(const ConvShape &s, const void *x, const void *w, void *y, hipStream_t st, const char **variant,
              const PostOp &post = PostOp(), void *split_ws = nullptr);
bool igemm_bwd_data_supported(const ConvShape &s);
size_t igemm_bwd_data_workspace(const ConvShape &s);   // bytes for the re-packed filter
size_t igemm_bwd_data_split_bytes(const ConvShape &s);   // scratch for a split reduction (0: never split)
// Filter preparation (re-pack per stride residue class / transpose of a 1x1 filter) into wt; a filter that the
// kernel reads in place is copied to wt only when copy_in_place_filter is set.
int igemm_bwd_data_prepare(const ConvShape &s, const void *w, void *wt, hipStream_t st, bool copy_in_place_filter);
int igemm_bwd_data(const ConvShape &s, const void *dy, const void *w_in_place, void *dx, const void *wt, hipStream_t st,
                   const char **variant, const PostOp &post = PostOp(), void *split_ws = nullptr);

// backward-data for C <= 4: G output columns form one GEMM row (see igemm.hip)
bool igemm_bwd_data_smallc_supported(const ConvShape &s);
void igemm_bwd_data_smallc_workspace(const ConvShape &s, size_t *w2_bytes, size_t *dx4_bytes);
int igemm_bwd_data_smallc_prepare(const ConvShape &s, const void *w, void *w2, hipStream_t st);
int igemm_bwd_data_smallc(const ConvShape &s, const void *dy, const void *w2, void *dx, void *dx4, hipStream_t st,
                          const char **variant, const PostOp &post = PostOp());

// names of the tile shapes the two MFMA kernel families are built in (nullptr past the last)
const char *igemm_tile_name(int index);
const char *igemm_stream_name(int index);   // names of the whole-launch kernels' plans (streaming kernel, window kernel)
// key (rows, output columns, reduction length) of the calling thread's last implicit-GEMM plan lookup
void igemm_last_plan_key(long long *M, int *Co, int *Kd);
const char *wgrad_tile_name(int index);

// ---- the implicit GEMM as its kernels see it (igemm.hip, stream.hip) ----------------------------------
constexpr int MAX_TAPS = 127;   // tap table capacity (11x11 = 121 fits)

// Out[m][co] = sum_{t,ci} In[pixel(m) + tap(t)][ci] * Wm[co][t*Ci + ci]; m runs over (image, row, column) of the
// launch's output grid, t over a TR x TS grid of filter taps, ci over the channels of a tap's contiguous run.
struct IgemmParams {
    const bf16_t *in;    // activations [N][Hi][Wi][Ci]
    const bf16_t *wm;    // filter matrix [Co][T*Ci]
    bf16_t *out;         // output tensor [N][Ho][Wo][Co]
    int N, Hi, Wi;
    int Ci;              // reduction elements per tap: a contiguous run starting at the tap's pixel
    int pix;             // elements per pixel in memory (== Ci for plain NHWC; smaller when a run spans pixels)
    int Co;
    int TR, TS, tstep_h, tstep_w;   // tap grid and the direction (+1 or -1) taps advance in, per axis
    int Mh, Mw;          // output grid of this launch (per image)
    int in_mul_h, in_mul_w, in_off_h, in_off_w;     // input coordinate of tap 0: a*in_mul + in_off
    int Ho, Wo, out_mul_h, out_mul_w, out_off_h, out_off_w;  // output coordinate: a*out_mul + out_off
    int linear_out;      // output pixel index == m (forward, and stride-1 backward-data)
    int M;               // N*Mh*Mw (< 2^31, checked by the launcher)
    int m_begin, m_end;  // GEMM rows [m_begin, m_end) belong to this launch (a problem may be cut in two launches of
                         // different tile shapes: see Plan); tile 0 starts at m_begin
    int m_tiles, n_tiles;
    unsigned in_bytes, wm_bytes;   // sizes of the two operand buffers (< 2^31)
    // BT kernels (1x1 stride-1 backward-data straight from the filter, no transposed copy): wm = w[K][Co];
    // reduction index k reads filter row k, whose Co output columns are contiguous.  Needs Ci % 64 == 0.
    unsigned bt_w_bytes; // size of the filter
    // split reduction (few tiles, long reduction): workgroup (tile, z) runs stages [z*split_stages, (z+1)*split_stages)
    // and stores its fp32 accumulators to partial[z][m][co]; a second kernel adds the splits in ascending z and
    // applies bias / ReLU / mask.  splits <= 1: off.
    float *partial;
    int splits, split_stages;
    int tap_row_inner;   // tap t = (column step)*TR + (row step) instead of (row step)*TS + (column step)
    int f32_out;         // store the fp32 accumulators to `partial` ([m][co], one split) instead of a rounded result to `out`
    int nt_out;          // the 16-byte result stores are non-temporal
    unsigned out_bytes;  // size of the output tensor when below 2 GiB (buffer stores with range-checked offsets), else 0
    int tap_inner;       // reduction order (Ci % BKT == 0 only): 1 = all taps of a channel block before the next block
    // applied to the accumulators before the store (all optional)
    const float *bias;   // + bias[co]
    int relu;            // max(0, .)
    const bf16_t *mask;  // indexed like `out`: the stored value is 0 where mask <= 0
};

// out[m][n] = sum_k a[m][k] * b[n][k] in fp32 from bf16 operands (k contiguous in both), on the tiled kernel
bool igemm_gemm_f32_supported(long long M, int Kd, int Nn);
int igemm_gemm_f32(long long M, int Kd, int Nn, const void *a, const void *b, float *out, hipStream_t st, const char **variant);

// ---- winograd.hip: 3x3 stride-1 forward in the transform domain, F(2x2, 3x3) ----------------------------
bool winograd_supported(const ConvShape &s);
// bytes of the three workspace parts: transformed filter U [16][K][C] bf16, transformed input V [16][tiles][C] bf16,
// products M [16][tiles][K] fp32
void winograd_workspace(const ConvShape &s, size_t *u_bytes, size_t *v_bytes, size_t *m_bytes);
int winograd_fwd(const ConvShape &s, const void *x, const void *w, void *y, void *u, void *v, void *m, hipStream_t st,
                 const char **variant, const PostOp &post);

// stream.hip: the same GEMM for short reductions and few output columns (see there); whether it can run p,
// and the launch over all rows (both take p as a launch site fills it: the fields the launcher derives -
// M, row range, tile counts, byte sizes, linear_out, tap_inner - are ignored and recomputed).
bool stream_applicable(const IgemmParams &p);
int stream_launch(const IgemmParams &p, hipStream_t st);
// window.hip: the same GEMM for multi-tap stride-1 layers of at most 64 input channels, from an LDS-resident input
// window and filter (see there); same conventions as the streaming kernel.
bool window_applicable(const IgemmParams &p);
int window_launch(const IgemmParams &p, hipStream_t st);

// ---- prep.hip: re-packing for channel counts that are not a multiple of 8 ---------
// [rows][C] -> [rows][C8] (C8 = C rounded up to 8, new channels zero); bf16 only.
int pad_channels(const void *src, void *dst, long long rows, int C, hipStream_t st);
// Small-C (C <= 4) image packing: `pix` channels per pixel, explicit zero border, padded size Hp x Wp;
// one filter row's taps form a contiguous run of `run` elements.
struct SmallCGeom { int pix, Hp, Wp, run; };
SmallCGeom smallc_geom(const ConvShape &s);
int smallc_pack_x(const ConvShape &s, const void *x, void *xp, hipStream_t st);   // xp: N*Hp*Wp*pix elements
int smallc_pack_w(const ConvShape &s, const void *w, void *wp, hipStream_t st);   // wp: K*R*run elements
// Space-to-depth (C <= 4, stride 2 or 4): s x s pixel blocks become channels of a stride-1 problem.
struct S2DGeom { int s, Cq, C2, R2, S2, H2, W2; };
S2DGeom s2d_geom(const ConvShape &s);
bool s2d_applicable(const ConvShape &s);
ConvShape s2d_shape(const ConvShape &s);      // the equivalent stride-1 problem: x2[N][H2][W2][C2], w2[K][R2][S2][C2]
int s2d_pack_x(const ConvShape &s, const void *x, void *x2, hipStream_t st);
int s2d_pack_w(const ConvShape &s, const void *w, void *w2, hipStream_t st);
int s2d_unpack_dx(const ConvShape &s, const void *dx2, void *dx, hipStream_t st, const void *mask = nullptr);   // mask: see PostOp
bool igemm_fwd_smallc_supported(const ConvShape &s);
int igemm_fwd_smallc(const ConvShape &s, const void *xp, const void *wp, void *y, hipStream_t st, const char **variant,
                     const PostOp &post = PostOp());

// ---- wgrad.hip: bf16 MFMA backward-weight with split reduction ------------------
// The problem as the kernel sees it: x[N][H][W][pix], dy[N][P][Q][K]; filter columns are TR*TS taps of
// `run` contiguous elements each; dw[k][r][s][c] (dense R,S,C) is read back from column
// r*col_r + s*col_s + c.
// With s2d > 1 the columns come from a space-to-depth problem: filter tap (r,s) sits in block
// (r/s2d, s/s2d) at channel ((r%s2d)*s2d + s%s2d)*Cq + c.
struct WgradGeom {
    int N, H, W, pix, K, P, Q, stride, pad, TR, TS, run, R, S, C, col_r, col_s, s2d, Cq;
    int oH, oW, ostride, opad;   // the caller's problem (with N, C, K, R, S: the key of the measured-plan table)
};
WgradGeom wgrad_geom_s2d(const ConvShape &s);       // x already packed by s2d_pack_x
WgradGeom wgrad_geom_plain(const ConvShape &s);     // C % 8 == 0
WgradGeom wgrad_geom_chanpad(const ConvShape &s);   // x already padded to C8 channels
WgradGeom wgrad_geom_smallc(const ConvShape &s);    // x already packed by smallc_pack_x
bool wgrad_supported(const WgradGeom &g);
size_t wgrad_workspace(const WgradGeom &g);            // bytes of fp32 partial tiles
// dw: fp32, or bf16 (the fp32 sum rounded once, by the reduce kernel) when dw_bf16
int wgrad(const WgradGeom &g, const void *x, const void *dy, void *dw, bool dw_bf16, float *partial, hipStream_t st,
          const char **variant);

}  // namespace mxc
