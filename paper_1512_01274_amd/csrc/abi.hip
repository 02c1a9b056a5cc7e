// C ABI entry points: argument validation, workspace carving, layout handling
// and kernel selection.  See include/mxc.h for the contract of every call.
#include <string.h>

#include <mutex>
#include <string>

#include "mxc_internal.h"

namespace mxc {

namespace {

thread_local char g_variant[128] = "";

void set_variant(const char *pass, const char *name)
{
    snprintf(g_variant, sizeof(g_variant), "%s:%s", pass, name);
}

// Sequential carve-out of the caller's workspace.  The same code path runs in
// "dry" mode (base == nullptr, nothing launched) to answer the size query, so
// the reported size is by construction what a real call consumes.
struct Carver {
    char *base;
    size_t used = 0;
    explicit Carver(void *b) : base((char *)b) {}
    void *take(size_t bytes)
    {
        const size_t off = used;
        used += align_up(bytes, 256);
        return base ? base + off : nullptr;
    }
};

int validate_shape(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                   ConvShape *out)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || R <= 0 || S <= 0 || stride <= 0 || pad < 0)
        return MXC_ERR_SHAPE;
    if ((long long)H + 2LL * pad < R || (long long)W + 2LL * pad < S) return MXC_ERR_SHAPE;
    if (dtype != MXC_F32 && dtype != MXC_BF16) return MXC_ERR_UNSUPPORTED;
    if (layout != MXC_NCHW && layout != MXC_NHWC) return MXC_ERR_UNSUPPORTED;
    ConvShape s{N, C, H, W, K, R, S, stride, pad, (H + 2 * pad - R) / stride + 1, (W + 2 * pad - S) / stride + 1};
    // Per-tensor element counts must stay below 2^40 (kernels index with 64 bits; this only
    // guards the size arithmetic) and the filter below 2^31 elements.
    const long double lim = 1099511627776.0L;
    if ((long double)N * C * H * W >= lim || (long double)N * K * s.P * s.Q >= lim ||
        (long double)K * C * R * S >= 2147483648.0L)
        return MXC_ERR_SHAPE;
    // NCHW operands are converted by batched transposes whose row and column counts are ints and whose grids
    // are bounded: refuse here, before anything is launched, what they could not run
    if (layout == MXC_NCHW) {
        const long long HW = (long long)H * W, PQ = (long long)s.P * s.Q, RS = (long long)R * S;
        if (!transpose_launchable(N, C, HW) || !transpose_launchable(N, HW, C) || !transpose_launchable(N, K, PQ) ||
            !transpose_launchable(N, PQ, K) || !transpose_launchable(K, C, RS) || !transpose_launchable(K, RS, C))
            return MXC_ERR_SHAPE;
    }
    *out = s;
    return MXC_OK;
}

bool misaligned(const void *p) { return ((uintptr_t)p & 15u) != 0; }

#define MXC_TRY(expr)                 \
    do {                              \
        const int rc_ = (expr);       \
        if (rc_ != MXC_OK) return rc_; \
    } while (0)

// ---- passes in the working layout (NHWC / KRSC) --------------------------------
// dry == true: only account workspace.

ConvShape with_channels(const ConvShape &s, int C)
{
    ConvShape t = s;
    t.C = C;
    return t;
}

// How forward and backward-weight get their input.  Layers whose channel count is not a multiple of 8 first
// bring x into the form their GEMM reads (space-to-depth packed, zero-bordered with 4 channels per pixel, or
// channel-padded), the same form for both passes; a caller that runs both on one x can have that done once
// (INPUT_PREPARE_ONLY fills a buffer of the caller's, nothing else runs) and hand the buffer to both
// (INPUT_PREPARED).  The form is carved from `xws` - the ordinary workspace in INPUT_RAW mode, the caller's
// buffer in the other two.  Layers that read x as it is have an empty prepared form.
enum InputMode { INPUT_RAW = 0, INPUT_PREPARE_ONLY = 1, INPUT_PREPARED = 2 };
enum InputForm { FORM_AS_IS = 0, FORM_S2D = 1, FORM_SMALLC = 2, FORM_CHANPAD = 3 };
struct InputPrep {
    Carver *xws = nullptr;
    InputMode mode = INPUT_RAW;
    int *form = nullptr;       // out: the InputForm the pass reads (the two passes must agree before they share a buffer)
};
inline void note_form(const InputPrep &ip, int form) { if (ip.form) *ip.form = form; }

int fwd_nhwc(const ConvShape &s, int dtype, const void *x, const void *w, void *y, const PostOp &post, Carver &ws, hipStream_t st,
             bool dry, const InputPrep &ip = InputPrep())
{
    const char *v = "";
    Carver &xws = ip.xws ? *ip.xws : ws;
    const bool pack = ip.mode != INPUT_PREPARED, run = ip.mode != INPUT_PREPARE_ONLY;
    if (dtype == MXC_BF16 && s.C % 8 == 0 && igemm_fwd_supported(s)) {
        const size_t split_bytes = run ? igemm_fwd_split_bytes(s) : 0;
        void *split_ws = split_bytes ? ws.take(split_bytes) : nullptr;
        if (dry || !run) return MXC_OK;
        const int rc = igemm_fwd(s, x, w, y, st, &v, post, split_ws);
        set_variant("fwd", v);
        return rc;
    }
    if (dtype == MXC_BF16 && s2d_applicable(s) && igemm_fwd_supported(s2d_shape(s))) {
        // strided first layer: space-to-depth turns it into a stride-1 problem with stride^2*C channels
        const ConvShape s2 = s2d_shape(s);
        note_form(ip, FORM_S2D);
        void *x2 = xws.take((size_t)s2.N * s2.H * s2.W * s2.C * 2);
        void *w2 = run ? ws.take((size_t)s2.K * s2.R * s2.S * s2.C * 2) : nullptr;
        if (dry) return MXC_OK;
        if (pack) MXC_TRY(s2d_pack_x(s, x, x2, st));
        if (!run) return MXC_OK;
        MXC_TRY(s2d_pack_w(s, w, w2, st));
        const int rc = igemm_fwd(s2, x2, w2, y, st, &v, post);
        set_variant("fwd", (std::string("s2d+") + v).c_str());
        return rc;
    }
    if (dtype == MXC_BF16 && s.C <= 4 && igemm_fwd_smallc_supported(s)) {
        // first-layer style: zero-bordered image with 4 or 8 channels per pixel, filter rows as runs
        const SmallCGeom g = smallc_geom(s);
        note_form(ip, FORM_SMALLC);
        void *xp = xws.take((size_t)s.N * g.Hp * g.Wp * g.pix * 2);
        void *wp = run ? ws.take((size_t)s.K * s.R * g.run * 2) : nullptr;
        if (dry) return MXC_OK;
        if (pack) MXC_TRY(smallc_pack_x(s, x, xp, st));
        if (!run) return MXC_OK;
        MXC_TRY(smallc_pack_w(s, w, wp, st));
        const int rc = igemm_fwd_smallc(s, xp, wp, y, st, &v, post);
        set_variant("fwd", (std::string("smallc+") + v).c_str());
        return rc;
    }
    const int C8 = (s.C + 7) / 8 * 8;
    if (dtype == MXC_BF16 && s.C % 8 != 0 && igemm_fwd_supported(with_channels(s, C8))) {
        // other channel counts: zero-pad the channels of x and w to a multiple of 8
        note_form(ip, FORM_CHANPAD);
        void *xp = xws.take((size_t)s.N * s.H * s.W * C8 * 2);
        void *wp = run ? ws.take((size_t)s.K * s.R * s.S * C8 * 2) : nullptr;
        if (dry) return MXC_OK;
        if (pack) MXC_TRY(pad_channels(x, xp, (long long)s.N * s.H * s.W, s.C, st));
        if (!run) return MXC_OK;
        MXC_TRY(pad_channels(w, wp, (long long)s.K * s.R * s.S, s.C, st));
        const int rc = igemm_fwd(with_channels(s, C8), xp, wp, y, st, &v, post);
        set_variant("fwd", (std::string("chanpad+") + v).c_str());
        return rc;
    }
    if (dry || !run) return MXC_OK;
    set_variant("fwd", "direct");
    return direct_fwd(s, dtype, x, w, y, st, post);
}

// How backward-data gets its filter.  Every bf16 path first brings the filter into the form its GEMM reads
// (re-packed per stride residue class, transposed, space-to-depth or column-group packed); a caller whose
// weights change less often than it calls backward-data can have that done once (FILTER_PREPARE_ONLY fills
// a buffer of the caller's, nothing else runs) and hand the buffer in afterwards (FILTER_PREPARED).  The
// prepared forms are carved from `fws` - the ordinary workspace in FILTER_RAW mode, the caller's buffer in
// the other two - in one fixed order, so all three modes agree on where each form lies.
enum FilterMode { FILTER_RAW = 0, FILTER_PREPARE_ONLY = 1, FILTER_PREPARED = 2 };

int bwd_data_nhwc(const ConvShape &s, int dtype, const void *dy, const void *w, void *dx, const PostOp &post, Carver &fws,
                  Carver &ws, hipStream_t st, bool dry, FilterMode mode = FILTER_RAW)
{
    const bool prep = mode != FILTER_PREPARED, run = mode != FILTER_PREPARE_ONLY;
    if (dtype == MXC_BF16 && s.K % 8 == 0 && s2d_applicable(s) && igemm_bwd_data_supported(s2d_shape(s))) {
        const ConvShape s2 = s2d_shape(s);
        void *w2 = fws.take((size_t)s2.K * s2.R * s2.S * s2.C * 2), *wt = fws.take(igemm_bwd_data_workspace(s2));
        void *dx2 = run ? ws.take((size_t)s2.N * s2.H * s2.W * s2.C * 2) : nullptr;
        if (dry) return MXC_OK;
        const char *v = "";
        if (prep) {
            MXC_TRY(s2d_pack_w(s, w, w2, st));
            MXC_TRY(igemm_bwd_data_prepare(s2, w2, wt, st, true));
        }
        if (!run) return MXC_OK;
        MXC_TRY(igemm_bwd_data(s2, dy, wt, dx2, wt, st, &v));
        set_variant("bwd_data", (std::string("s2d+") + v).c_str());
        return s2d_unpack_dx(s, dx2, dx, st, post.mask);      // the mask is applied where dx itself is written
    }
    if (dtype == MXC_BF16 && igemm_bwd_data_smallc_supported(s)) {
        size_t w2_bytes, dx4_bytes;
        igemm_bwd_data_smallc_workspace(s, &w2_bytes, &dx4_bytes);
        void *w2 = fws.take(w2_bytes), *dx4 = run ? ws.take(dx4_bytes) : nullptr;
        if (dry) return MXC_OK;
        const char *v = "";
        if (prep) MXC_TRY(igemm_bwd_data_smallc_prepare(s, w, w2, st));
        if (!run) return MXC_OK;
        const int rc = igemm_bwd_data_smallc(s, dy, w2, dx, dx4, st, &v, post);
        set_variant("bwd_data", (std::string("smallc+") + v).c_str());
        return rc;
    }
    if (dtype == MXC_BF16 && igemm_bwd_data_supported(s)) {
        void *wt = fws.take(igemm_bwd_data_workspace(s));
        const size_t split_bytes = run ? igemm_bwd_data_split_bytes(s) : 0;
        void *split_ws = split_bytes ? ws.take(split_bytes) : nullptr;
        if (dry) return MXC_OK;
        const char *v = "";
        // a filter the kernel reads in place stays where it is unless the caller keeps a prepared copy
        if (prep) MXC_TRY(igemm_bwd_data_prepare(s, w, wt, st, mode == FILTER_PREPARE_ONLY));
        if (!run) return MXC_OK;
        const int rc = igemm_bwd_data(s, dy, mode == FILTER_RAW ? w : wt, dx, wt, st, &v, post, split_ws);
        set_variant("bwd_data", v);
        return rc;
    }
    // direct kernels read the KRSC filter itself: its prepared form is a copy
    const size_t wbytes = (size_t)s.K * s.R * s.S * s.C * elem_size(dtype);
    void *wc = mode != FILTER_RAW ? fws.take(wbytes) : nullptr;
    if (dry) return MXC_OK;
    if (mode == FILTER_PREPARE_ONLY) return launch_copy(w, wc, wbytes, st);
    set_variant("bwd_data", "direct");
    return direct_bwd_data(s, dtype, dy, mode == FILTER_PREPARED ? wc : w, dx, st, post);
}

// ip: see InputMode (the forms are those of fwd_nhwc, chosen by the same tests in the same order; only
// INPUT_RAW and INPUT_PREPARED reach this function)
int bwd_weight_nhwc(const ConvShape &s, int dtype, const void *x, const void *dy, void *dw, bool dw_bf16, Carver &ws,
                    hipStream_t st, bool dry, const InputPrep &ip = InputPrep())
{
    const char *v = "";
    Carver &xws = ip.xws ? *ip.xws : ws;
    const bool pack = ip.mode != INPUT_PREPARED;
    if (dtype == MXC_BF16 && s.C % 8 == 0 && wgrad_supported(wgrad_geom_plain(s))) {
        const WgradGeom g = wgrad_geom_plain(s);
        float *partial = (float *)ws.take(wgrad_workspace(g));
        if (dry) return MXC_OK;
        const int rc = wgrad(g, x, dy, dw, dw_bf16, partial, st, &v);
        set_variant("bwd_weight", v);
        return rc;
    }
    if (dtype == MXC_BF16 && s2d_applicable(s) && wgrad_supported(wgrad_geom_s2d(s))) {
        const ConvShape s2 = s2d_shape(s);
        const WgradGeom g = wgrad_geom_s2d(s);
        note_form(ip, FORM_S2D);
        void *x2 = xws.take((size_t)s2.N * s2.H * s2.W * s2.C * 2);
        float *partial = (float *)ws.take(wgrad_workspace(g));
        if (dry) return MXC_OK;
        if (pack) MXC_TRY(s2d_pack_x(s, x, x2, st));
        const int rc = wgrad(g, x2, dy, dw, dw_bf16, partial, st, &v);
        set_variant("bwd_weight", (std::string("s2d+") + v).c_str());
        return rc;
    }
    if (dtype == MXC_BF16 && s.C <= 4 && wgrad_supported(wgrad_geom_smallc(s))) {
        const SmallCGeom sg = smallc_geom(s);
        const WgradGeom g = wgrad_geom_smallc(s);
        note_form(ip, FORM_SMALLC);
        void *xp = xws.take((size_t)s.N * sg.Hp * sg.Wp * sg.pix * 2);
        float *partial = (float *)ws.take(wgrad_workspace(g));
        if (dry) return MXC_OK;
        if (pack) MXC_TRY(smallc_pack_x(s, x, xp, st));
        const int rc = wgrad(g, xp, dy, dw, dw_bf16, partial, st, &v);
        set_variant("bwd_weight", (std::string("smallc+") + v).c_str());
        return rc;
    }
    if (dtype == MXC_BF16 && s.C % 8 != 0 && wgrad_supported(wgrad_geom_chanpad(s))) {
        const WgradGeom g = wgrad_geom_chanpad(s);
        note_form(ip, FORM_CHANPAD);
        void *xp = xws.take((size_t)s.N * s.H * s.W * g.pix * 2);
        float *partial = (float *)ws.take(wgrad_workspace(g));
        if (dry) return MXC_OK;
        if (pack) MXC_TRY(pad_channels(x, xp, (long long)s.N * s.H * s.W, s.C, st));
        const int rc = wgrad(g, xp, dy, dw, dw_bf16, partial, st, &v);
        set_variant("bwd_weight", (std::string("chanpad+") + v).c_str());
        return rc;
    }
    const int splits = direct_bwd_weight_splits(s);
    float *partial = (float *)ws.take((size_t)splits * s.K * s.R * s.S * s.C * sizeof(float));
    if (dry) return MXC_OK;
    set_variant("bwd_weight", "direct_splitk");
    return direct_bwd_weight(s, dtype, x, dy, dw, dw_bf16, partial, splits, st);
}

// ---- one driver per pass: handles the caller's layout ---------------------------

// fws / mode: see FilterMode (backward-data only; fws == ws and FILTER_RAW otherwise)
int run_pass(int pass, const ConvShape &s, int dtype, int layout, const void *a, const void *b, void *out, const PostOp &post,
             Carver &ws, hipStream_t st, bool dry, Carver *fws_opt = nullptr, FilterMode mode = FILTER_RAW)
{
    Carver &fws = fws_opt ? *fws_opt : ws;
    const int eb = (int)elem_size(dtype);
    const size_t nx = (size_t)s.N * s.C * s.H * s.W, nw = (size_t)s.K * s.C * s.R * s.S,
                 ny = (size_t)s.N * s.K * s.P * s.Q;
    if (layout == MXC_NHWC) {
        switch (pass) {
        case MXC_FWD: return fwd_nhwc(s, dtype, a, b, out, post, ws, st, dry);
        case MXC_BWD_DATA: return bwd_data_nhwc(s, dtype, a, b, out, post, fws, ws, st, dry, mode);
        default: return bwd_weight_nhwc(s, dtype, a, b, out, pass == MXC_BWD_WEIGHT_BF16, ws, st, dry);
        }
    }
    // NCHW at the boundary: convert operands into the workspace, compute, convert the result back.
    if (pass == MXC_FWD) {
        void *x2 = ws.take(nx * eb), *w2 = ws.take(nw * eb), *y2 = ws.take(ny * eb);
        if (!dry) {
            MXC_TRY(launch_transpose(a, x2, s.N, s.C, s.H * s.W, eb, st));
            MXC_TRY(launch_transpose(b, w2, s.K, s.C, s.R * s.S, eb, st));
        }
        MXC_TRY(fwd_nhwc(s, dtype, x2, w2, y2, post, ws, st, dry));
        if (!dry) MXC_TRY(launch_transpose(y2, out, s.N, s.P * s.Q, s.K, eb, st));
        return MXC_OK;
    }
    if (pass == MXC_BWD_DATA) {
        const bool prep = mode != FILTER_PREPARED, run = mode != FILTER_PREPARE_ONLY;
        void *w2 = fws.take(nw * eb);      // the KRSC filter is the first of the prepared forms
        void *dy2 = run ? ws.take(ny * eb) : nullptr, *dx2 = run ? ws.take(nx * eb) : nullptr;
        // with_mask (not the pointer) decides the carve-out, so that the size query and the call agree
        void *mask2 = run && (post.mask != nullptr || post.relu) ? ws.take(nx * eb) : nullptr;
        PostOp post2 = post;
        post2.relu = 0;
        if (!dry) {
            if (run) MXC_TRY(launch_transpose(a, dy2, s.N, s.K, s.P * s.Q, eb, st));
            if (prep) MXC_TRY(launch_transpose(b, w2, s.K, s.C, s.R * s.S, eb, st));
            if (run && post.mask != nullptr) {
                MXC_TRY(launch_transpose(post.mask, mask2, s.N, s.C, s.H * s.W, eb, st));
                post2.mask = mask2;
            }
        }
        MXC_TRY(bwd_data_nhwc(s, dtype, dy2, w2, dx2, post2, fws, ws, st, dry, mode));
        if (!dry && run) MXC_TRY(launch_transpose(dx2, out, s.N, s.H * s.W, s.C, eb, st));
        return MXC_OK;
    }
    const bool dw_bf16 = pass == MXC_BWD_WEIGHT_BF16;
    const int dwb = dw_bf16 ? 2 : 4;
    void *x2 = ws.take(nx * eb), *dy2 = ws.take(ny * eb);
    void *dw2 = ws.take(nw * dwb);
    if (!dry) {
        MXC_TRY(launch_transpose(a, x2, s.N, s.C, s.H * s.W, eb, st));
        MXC_TRY(launch_transpose(b, dy2, s.N, s.K, s.P * s.Q, eb, st));
    }
    MXC_TRY(bwd_weight_nhwc(s, dtype, x2, dy2, dw2, dw_bf16, ws, st, dry));
    if (!dry) MXC_TRY(launch_transpose(dw2, out, s.K, s.R * s.S, s.C, dwb, st));
    return MXC_OK;
}

// `post.relu` doubles, for backward-data in dry runs, as "a mask will be given" (the mask pointer is
// not known to the size query).
int entry(int pass, int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
          const void *a, const void *b, void *out, const PostOp &post, void *workspace, size_t workspace_bytes,
          void *hip_stream)
{
    ConvShape s;
    MXC_TRY(validate_shape(N, C, H, W, K, R, S, stride, pad, dtype, layout, &s));
    if (!a || !b || !out) return MXC_ERR_NULL;
    if (misaligned(a) || misaligned(b) || misaligned(out) || misaligned(workspace) || misaligned(post.mask)) return MXC_ERR_ALIGN;
    Carver need(nullptr);
    PostOp dry_post;
    dry_post.relu = (post.mask != nullptr || post.relu) ? 1 : 0;
    MXC_TRY(run_pass(pass, s, dtype, layout, nullptr, nullptr, nullptr, dry_post, need, nullptr, true));
    if (need.used > 0 && (!workspace || workspace_bytes < need.used)) return MXC_ERR_WORKSPACE;
    Carver ws(workspace);
    return run_pass(pass, s, dtype, layout, a, b, out, post, ws, (hipStream_t)hip_stream, false);
}

}  // namespace
}  // namespace mxc

// ---- scratch of the entry point that allocates nothing ------------------------------------------
// One array per GPU, part of the loaded code object: it exists on every device the library runs on
// from the first use of the library there until the process ends.  In host code the name below is
// only a handle for hipGetSymbolAddress; kernels and copies get the device address it returns.
#define MXC_STATIC_SCRATCH_BYTES (64u << 20)
static __device__ __align__(256) unsigned char scratch[MXC_STATIC_SCRATCH_BYTES];

namespace mxc {
namespace {

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES] = {};

// Device address of `scratch` on the current device (looked up once per device, with that device current).
int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return MXC_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return MXC_ERR_LAUNCH;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return MXC_OK;
}

}  // namespace
}  // namespace mxc

using namespace mxc;

extern "C" {

int mxc_conv2d_fwd(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                   const void *x, const void *w, void *y, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return entry(MXC_FWD, N, C, H, W, K, R, S, stride, pad, dtype, layout, x, w, y, PostOp(), workspace, workspace_bytes,
                 hip_stream);
}

int mxc_conv2d_bwd_data(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                        const void *dy, const void *w, void *dx, void *workspace, size_t workspace_bytes,
                        void *hip_stream)
{
    return entry(MXC_BWD_DATA, N, C, H, W, K, R, S, stride, pad, dtype, layout, dy, w, dx, PostOp(), workspace, workspace_bytes,
                 hip_stream);
}

int mxc_conv2d_bwd_weight(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                          const void *x, const void *dy, void *dw, void *workspace, size_t workspace_bytes,
                          void *hip_stream)
{
    return entry(MXC_BWD_WEIGHT, N, C, H, W, K, R, S, stride, pad, dtype, layout, x, dy, dw, PostOp(), workspace,
                 workspace_bytes, hip_stream);
}

int mxc_conv2d_bwd_weight_bf16(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                               const void *x, const void *dy, void *dw, void *workspace, size_t workspace_bytes,
                               void *hip_stream)
{
    if (dtype != MXC_BF16) return MXC_ERR_UNSUPPORTED;
    return entry(MXC_BWD_WEIGHT_BF16, N, C, H, W, K, R, S, stride, pad, dtype, layout, x, dy, dw, PostOp(), workspace,
                 workspace_bytes, hip_stream);
}

int mxc_conv2d_bwd_weight_static(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                                 const void *x, const void *dy, void *dw, void *hip_stream)
{
    // argument errors first, as the other entry points report them; then the size against the array
    ConvShape s;
    MXC_TRY(validate_shape(N, C, H, W, K, R, S, stride, pad, dtype, layout, &s));
    if (!x || !dy || !dw) return MXC_ERR_NULL;
    if (misaligned(x) || misaligned(dy) || misaligned(dw)) return MXC_ERR_ALIGN;
    Carver need(nullptr);
    MXC_TRY(run_pass(MXC_BWD_WEIGHT, s, dtype, layout, nullptr, nullptr, nullptr, PostOp(), need, nullptr, true));
    if (need.used > MXC_STATIC_SCRATCH_BYTES) return MXC_ERR_WORKSPACE;
    void *ws = nullptr;
    MXC_TRY(static_scratch(&ws));
    // every kernel of this pass writes the part of the scratch it later reads: nothing needs clearing
    return entry(MXC_BWD_WEIGHT, N, C, H, W, K, R, S, stride, pad, dtype, layout, x, dy, dw, PostOp(), ws, MXC_STATIC_SCRATCH_BYTES,
                 hip_stream);
}

int mxc_conv2d_fwd_bias_act(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                            const void *x, const void *w, const float *bias, int relu, void *y, void *workspace,
                            size_t workspace_bytes, void *hip_stream)
{
    if (relu != 0 && relu != 1) return MXC_ERR_UNSUPPORTED;
    if (bias != nullptr && ((uintptr_t)bias & 3u)) return MXC_ERR_ALIGN;
    PostOp post;
    post.bias = bias;
    post.relu = relu;
    // the forward pass's workspace does not depend on the grouped operations: query it as MXC_FWD
    ConvShape s;
    MXC_TRY(validate_shape(N, C, H, W, K, R, S, stride, pad, dtype, layout, &s));
    if (!x || !w || !y) return MXC_ERR_NULL;
    if (misaligned(x) || misaligned(w) || misaligned(y) || misaligned(workspace)) return MXC_ERR_ALIGN;
    Carver need(nullptr);
    MXC_TRY(run_pass(MXC_FWD, s, dtype, layout, nullptr, nullptr, nullptr, PostOp(), need, nullptr, true));
    if (need.used > 0 && (!workspace || workspace_bytes < need.used)) return MXC_ERR_WORKSPACE;
    Carver ws(workspace);
    return run_pass(MXC_FWD, s, dtype, layout, x, w, y, post, ws, (hipStream_t)hip_stream, false);
}

int mxc_conv2d_bwd_data_relu(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                             const void *dy, const void *w, const void *x, void *dx, void *workspace, size_t workspace_bytes,
                             void *hip_stream)
{
    if (!x) return MXC_ERR_NULL;
    PostOp post;
    post.mask = x;
    return entry(MXC_BWD_DATA, N, C, H, W, K, R, S, stride, pad, dtype, layout, dy, w, dx, post, workspace, workspace_bytes,
                 hip_stream);
}

int mxc_conv2d_bwd_data_prepare_filter(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                                       const void *w, void *w_prepared, size_t prepared_bytes, void *hip_stream)
{
    ConvShape s;
    MXC_TRY(validate_shape(N, C, H, W, K, R, S, stride, pad, dtype, layout, &s));
    if (!w || !w_prepared) return MXC_ERR_NULL;
    if (misaligned(w) || misaligned(w_prepared)) return MXC_ERR_ALIGN;
    Carver need(nullptr), none(nullptr);
    MXC_TRY(run_pass(MXC_BWD_DATA, s, dtype, layout, nullptr, nullptr, nullptr, PostOp(), none, nullptr, true, &need, FILTER_PREPARE_ONLY));
    if (prepared_bytes < need.used) return MXC_ERR_WORKSPACE;
    Carver fws(w_prepared);
    return run_pass(MXC_BWD_DATA, s, dtype, layout, nullptr, w, nullptr, PostOp(), none, (hipStream_t)hip_stream, false, &fws,
                    FILTER_PREPARE_ONLY);
}

int mxc_conv2d_bwd_data_prepared(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                                 const void *dy, const void *w_prepared, size_t prepared_bytes, const void *x_mask, void *dx,
                                 void *workspace, size_t workspace_bytes, void *hip_stream)
{
    ConvShape s;
    MXC_TRY(validate_shape(N, C, H, W, K, R, S, stride, pad, dtype, layout, &s));
    if (!dy || !w_prepared || !dx) return MXC_ERR_NULL;
    if (misaligned(dy) || misaligned(w_prepared) || misaligned(dx) || misaligned(workspace) || misaligned(x_mask)) return MXC_ERR_ALIGN;
    PostOp post, dry_post;
    post.mask = x_mask;
    dry_post.relu = x_mask != nullptr ? 1 : 0;
    Carver needf(nullptr), need(nullptr);
    MXC_TRY(run_pass(MXC_BWD_DATA, s, dtype, layout, nullptr, nullptr, nullptr, dry_post, need, nullptr, true, &needf, FILTER_PREPARED));
    if (prepared_bytes < needf.used) return MXC_ERR_WORKSPACE;
    if (need.used > 0 && (!workspace || workspace_bytes < need.used)) return MXC_ERR_WORKSPACE;
    Carver fws(const_cast<void *>(w_prepared)), ws(workspace);
    return run_pass(MXC_BWD_DATA, s, dtype, layout, dy, nullptr, dx, post, ws, (hipStream_t)hip_stream, false, &fws, FILTER_PREPARED);
}

namespace mxc {
namespace {

// Size and kind of the prepared input of a layer.  Forward and backward-weight must read the same form to share
// a buffer; for a shape where they would not (one of them falls back to another kernel family) the prepared
// form is empty, like that of a layer that reads x as it is, and each pass packs for itself as usual.
int prepared_input_plan(const ConvShape &s, int dtype, size_t *bytes, int *form)
{
    Carver none(nullptr), xf(nullptr), xw(nullptr);
    int form_f = FORM_AS_IS, form_w = FORM_AS_IS;
    InputPrep ipf, ipw;
    ipf.xws = &xf; ipf.mode = INPUT_PREPARE_ONLY; ipf.form = &form_f;
    ipw.xws = &xw; ipw.mode = INPUT_PREPARED; ipw.form = &form_w;
    MXC_TRY(fwd_nhwc(s, dtype, nullptr, nullptr, nullptr, PostOp(), none, nullptr, true, ipf));
    MXC_TRY(bwd_weight_nhwc(s, dtype, nullptr, nullptr, nullptr, false, none, nullptr, true, ipw));
    const bool shared = form_f == form_w && xf.used == xw.used;
    *bytes = shared ? xf.used : 0;
    *form = shared ? form_f : FORM_AS_IS;
    return MXC_OK;
}

}  // namespace
}  // namespace mxc

int mxc_conv2d_prepare_input(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                             const void *x, void *x_prepared, size_t prepared_bytes, void *hip_stream)
{
    ConvShape s;
    MXC_TRY(validate_shape(N, C, H, W, K, R, S, stride, pad, dtype, layout, &s));
    if (layout != MXC_NHWC) return MXC_ERR_UNSUPPORTED;
    if (!x) return MXC_ERR_NULL;
    if (misaligned(x) || misaligned(x_prepared)) return MXC_ERR_ALIGN;
    size_t need = 0;
    int form = FORM_AS_IS;
    MXC_TRY(prepared_input_plan(s, dtype, &need, &form));
    if (need == 0) return MXC_OK;          // the layer reads x as it is
    if (!x_prepared) return MXC_ERR_NULL;
    if (prepared_bytes < need) return MXC_ERR_WORKSPACE;
    Carver none(nullptr), xws(x_prepared);
    InputPrep ip;
    ip.xws = &xws; ip.mode = INPUT_PREPARE_ONLY;
    return fwd_nhwc(s, dtype, x, nullptr, nullptr, PostOp(), none, (hipStream_t)hip_stream, false, ip);
}

int mxc_conv2d_fwd_prepared_input(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                                  const void *x_prepared, size_t prepared_bytes, const void *w, const float *bias, int relu,
                                  void *y, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    ConvShape s;
    MXC_TRY(validate_shape(N, C, H, W, K, R, S, stride, pad, dtype, layout, &s));
    if (layout != MXC_NHWC || (relu != 0 && relu != 1)) return MXC_ERR_UNSUPPORTED;
    if (!x_prepared || !w || !y) return MXC_ERR_NULL;
    if (misaligned(x_prepared) || misaligned(w) || misaligned(y) || misaligned(workspace) || ((uintptr_t)bias & 3u)) return MXC_ERR_ALIGN;
    size_t needx = 0;
    int form = FORM_AS_IS;
    MXC_TRY(prepared_input_plan(s, dtype, &needx, &form));
    if (prepared_bytes < needx) return MXC_ERR_WORKSPACE;
    PostOp post;
    post.bias = bias;
    post.relu = relu;
    InputPrep ip;
    Carver need(nullptr), nx(nullptr);
    if (needx) { ip.xws = &nx; ip.mode = INPUT_PREPARED; }
    MXC_TRY(fwd_nhwc(s, dtype, nullptr, nullptr, nullptr, PostOp(), need, nullptr, true, ip));
    if (need.used > 0 && (!workspace || workspace_bytes < need.used)) return MXC_ERR_WORKSPACE;
    Carver ws(workspace), xws(const_cast<void *>(x_prepared));
    if (needx) ip.xws = &xws;
    // an empty prepared form: x_prepared is x itself
    return fwd_nhwc(s, dtype, needx ? nullptr : x_prepared, w, y, post, ws, (hipStream_t)hip_stream, false, ip);
}

int mxc_conv2d_bwd_weight_prepared_input(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype,
                                         int layout, const void *x_prepared, size_t prepared_bytes, const void *dy, void *dw,
                                         int dw_dtype, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    ConvShape s;
    MXC_TRY(validate_shape(N, C, H, W, K, R, S, stride, pad, dtype, layout, &s));
    if (layout != MXC_NHWC || (dw_dtype != MXC_F32 && dw_dtype != MXC_BF16) || (dw_dtype == MXC_BF16 && dtype != MXC_BF16))
        return MXC_ERR_UNSUPPORTED;
    if (!x_prepared || !dy || !dw) return MXC_ERR_NULL;
    if (misaligned(x_prepared) || misaligned(dy) || misaligned(dw) || misaligned(workspace)) return MXC_ERR_ALIGN;
    size_t needx = 0;
    int form = FORM_AS_IS;
    MXC_TRY(prepared_input_plan(s, dtype, &needx, &form));
    if (prepared_bytes < needx) return MXC_ERR_WORKSPACE;
    InputPrep ip;
    Carver need(nullptr), nx(nullptr);
    if (needx) { ip.xws = &nx; ip.mode = INPUT_PREPARED; }
    MXC_TRY(bwd_weight_nhwc(s, dtype, nullptr, nullptr, nullptr, dw_dtype == MXC_BF16, need, nullptr, true, ip));
    if (need.used > 0 && (!workspace || workspace_bytes < need.used)) return MXC_ERR_WORKSPACE;
    Carver ws(workspace), xws(const_cast<void *>(x_prepared));
    if (needx) ip.xws = &xws;
    return bwd_weight_nhwc(s, dtype, needx ? nullptr : x_prepared, dy, dw, dw_dtype == MXC_BF16, ws, (hipStream_t)hip_stream, false, ip);
}

int mxc_conv2d_fwd_transform(int N, int C, int H, int W, int K, int R, int S, int stride, int pad, int dtype, int layout,
                             const void *x, const void *w, const float *bias, int relu, void *y, void *workspace,
                             size_t workspace_bytes, void *hip_stream)
{
    ConvShape s;
    MXC_TRY(validate_shape(N, C, H, W, K, R, S, stride, pad, dtype, layout, &s));
    if (dtype != MXC_BF16 || layout != MXC_NHWC || (relu != 0 && relu != 1) || !winograd_supported(s)) return MXC_ERR_UNSUPPORTED;
    if (!x || !w || !y) return MXC_ERR_NULL;
    if (misaligned(x) || misaligned(w) || misaligned(y) || misaligned(workspace) || ((uintptr_t)bias & 3u)) return MXC_ERR_ALIGN;
    size_t ub, vb, mb;
    winograd_workspace(s, &ub, &vb, &mb);
    Carver need(nullptr);
    need.take(ub); need.take(vb); need.take(mb);
    if (!workspace || workspace_bytes < need.used) return MXC_ERR_WORKSPACE;
    Carver ws(workspace);
    void *u = ws.take(ub), *v = ws.take(vb), *m = ws.take(mb);
    PostOp post;
    post.bias = bias;
    post.relu = relu;
    const char *vname = "";
    const int rc = winograd_fwd(s, x, w, y, u, v, m, (hipStream_t)hip_stream, &vname, post);
    if (rc == MXC_OK) set_variant("fwd", vname);
    return rc;
}

int mxc_bias_grad(int N, int K, int P, int Q, int dtype, int layout, const void *dy, float *db, void *workspace,
                  size_t workspace_bytes, void *hip_stream)
{
    if (N <= 0 || K <= 0 || P <= 0 || Q <= 0) return MXC_ERR_SHAPE;
    if ((long double)N * K * P * Q >= 1099511627776.0L) return MXC_ERR_SHAPE;
    if (dtype != MXC_F32 && dtype != MXC_BF16) return MXC_ERR_UNSUPPORTED;
    if (layout != MXC_NCHW && layout != MXC_NHWC) return MXC_ERR_UNSUPPORTED;
    if (!dy || !db) return MXC_ERR_NULL;
    if (misaligned(dy) || misaligned(db) || misaligned(workspace)) return MXC_ERR_ALIGN;
    const size_t need = (size_t)bias_grad_parts(N, K, (long long)P * Q, layout) * K * sizeof(float);
    if (!workspace || workspace_bytes < need) return MXC_ERR_WORKSPACE;
    return bias_grad(N, K, (long long)P * Q, dtype, layout, dy, db, (float *)workspace, (hipStream_t)hip_stream);
}

int mxc_fc_fwd(int N, int C, int K, int dtype, const void *x, const void *w, const float *bias, int relu, void *y,
               void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return mxc_conv2d_fwd_bias_act(N, C, 1, 1, K, 1, 1, 1, 0, dtype, MXC_NHWC, x, w, bias, relu, y, workspace, workspace_bytes,
                                   hip_stream);
}

int mxc_fc_bwd_data(int N, int C, int K, int dtype, const void *dy, const void *w, const void *x_mask, void *dx,
                    void *workspace, size_t workspace_bytes, void *hip_stream)
{
    PostOp post;
    post.mask = x_mask;
    return entry(MXC_BWD_DATA, N, C, 1, 1, K, 1, 1, 1, 0, dtype, MXC_NHWC, dy, w, dx, post, workspace, workspace_bytes, hip_stream);
}

int mxc_fc_bwd_weight(int N, int C, int K, int dtype, const void *x, const void *dy, void *dw,
                      void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return mxc_conv2d_bwd_weight(N, C, 1, 1, K, 1, 1, 1, 0, dtype, MXC_NHWC, x, dy, dw, workspace, workspace_bytes, hip_stream);
}

int mxc_softmax_fwd(int N, int K, int dtype, const void *z, void *p, void *hip_stream)
{
    if (N <= 0 || K <= 0) return MXC_ERR_SHAPE;
    if (dtype != MXC_F32 && dtype != MXC_BF16) return MXC_ERR_UNSUPPORTED;
    if (!z || !p) return MXC_ERR_NULL;
    if (misaligned(z) || misaligned(p)) return MXC_ERR_ALIGN;
    return softmax_fwd(N, K, dtype, z, p, (hipStream_t)hip_stream);
}

int mxc_softmax_xent_bwd(int N, int K, int dtype, const void *p, const int *labels, float scale, void *dz, void *hip_stream)
{
    if (N <= 0 || K <= 0) return MXC_ERR_SHAPE;
    if (dtype != MXC_F32 && dtype != MXC_BF16) return MXC_ERR_UNSUPPORTED;
    if (!p || !labels || !dz) return MXC_ERR_NULL;
    if (misaligned(p) || misaligned(dz) || ((uintptr_t)labels & 3u)) return MXC_ERR_ALIGN;
    return softmax_xent_bwd(N, K, dtype, p, labels, dz, scale, (hipStream_t)hip_stream);
}

int mxc_sgd_update(size_t n, float *w, const float *g, float *v, void *w_bf16, float lr, float momentum, float wd, void *hip_stream)
{
    if (n == 0) return MXC_ERR_SHAPE;
    if (!w || !g) return MXC_ERR_NULL;
    if (!v && momentum != 0.f) return MXC_ERR_NULL;
    if (misaligned(w) || misaligned(g) || misaligned(v) || misaligned(w_bf16)) return MXC_ERR_ALIGN;
    return sgd_update(n, w, g, v, w_bf16, lr, momentum, wd, (hipStream_t)hip_stream);
}

int mxc_conv2d_workspace_bytes(int pass, int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                               int dtype, int layout, size_t *out_bytes)
{
    if (!out_bytes) return MXC_ERR_NULL;
    if (pass < MXC_FWD || pass > MXC_FWD_TRANSFORM) return MXC_ERR_UNSUPPORTED;
    if (pass == MXC_BWD_WEIGHT_BF16 && dtype != MXC_BF16) return MXC_ERR_UNSUPPORTED;
    ConvShape s;
    const int rc = validate_shape(N, C, H, W, K, R, S, stride, pad, dtype, layout, &s);
    if (rc != MXC_OK) return rc;
    if (pass == MXC_BIAS_GRAD) {
        *out_bytes = align_up((size_t)bias_grad_parts(s.N, s.K, (long long)s.P * s.Q, layout) * s.K * sizeof(float), 256);
        return MXC_OK;
    }
    if (pass == MXC_FWD_TRANSFORM) {
        if (dtype != MXC_BF16 || layout != MXC_NHWC || !winograd_supported(s)) return MXC_ERR_UNSUPPORTED;
        size_t ub, vb, mb;
        winograd_workspace(s, &ub, &vb, &mb);
        Carver need(nullptr);
        need.take(ub); need.take(vb); need.take(mb);
        *out_bytes = need.used;
        return MXC_OK;
    }
    if (pass >= MXC_INPUT_PREPARED) {
        if (layout != MXC_NHWC || (pass == MXC_BWD_WEIGHT_PREPARED_INPUT_BF16 && dtype != MXC_BF16)) return MXC_ERR_UNSUPPORTED;
        size_t needx = 0;
        int form = FORM_AS_IS;
        MXC_TRY(prepared_input_plan(s, dtype, &needx, &form));
        if (pass == MXC_INPUT_PREPARED) { *out_bytes = needx; return MXC_OK; }
        InputPrep ip;
        Carver needw(nullptr), nx(nullptr);
        if (needx) { ip.xws = &nx; ip.mode = INPUT_PREPARED; }
        if (pass == MXC_FWD_PREPARED_INPUT) MXC_TRY(fwd_nhwc(s, dtype, nullptr, nullptr, nullptr, PostOp(), needw, nullptr, true, ip));
        else MXC_TRY(bwd_weight_nhwc(s, dtype, nullptr, nullptr, nullptr, pass == MXC_BWD_WEIGHT_PREPARED_INPUT_BF16, needw, nullptr, true, ip));
        *out_bytes = needw.used;
        return MXC_OK;
    }
    Carver need(nullptr), needf(nullptr);
    PostOp dry_post;
    dry_post.relu = pass == MXC_BWD_DATA_RELU || pass == MXC_BWD_DATA_PREPARED_RELU;
    if (pass == MXC_BWD_DATA_FILTER || pass == MXC_BWD_DATA_PREPARED || pass == MXC_BWD_DATA_PREPARED_RELU) {
        const FilterMode mode = pass == MXC_BWD_DATA_FILTER ? FILTER_PREPARE_ONLY : FILTER_PREPARED;
        const int rc3 = run_pass(MXC_BWD_DATA, s, dtype, layout, nullptr, nullptr, nullptr, dry_post, need, nullptr, true, &needf, mode);
        if (rc3 != MXC_OK) return rc3;
        *out_bytes = pass == MXC_BWD_DATA_FILTER ? needf.used : need.used;
        return MXC_OK;
    }
    const int rc2 = run_pass(pass == MXC_BWD_DATA_RELU ? MXC_BWD_DATA : pass, s, dtype, layout, nullptr, nullptr, nullptr, dry_post,
                             need, nullptr, true);
    if (rc2 != MXC_OK) return rc2;
    *out_bytes = need.used;
    return MXC_OK;
}

int mxc_layout_convert(int n, int c, int h, int w, int dtype, int src_layout, int dst_layout, const void *src,
                       void *dst, void *hip_stream)
{
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0) return MXC_ERR_SHAPE;
    if ((long double)n * c * h * w >= 1099511627776.0L || !transpose_launchable(n, c, (long long)h * w) ||
        !transpose_launchable(n, (long long)h * w, c))
        return MXC_ERR_SHAPE;
    if (dtype != MXC_F32 && dtype != MXC_BF16) return MXC_ERR_UNSUPPORTED;
    if ((src_layout != MXC_NCHW && src_layout != MXC_NHWC) || (dst_layout != MXC_NCHW && dst_layout != MXC_NHWC))
        return MXC_ERR_UNSUPPORTED;
    if (!src || !dst) return MXC_ERR_NULL;
    if (misaligned(src) || misaligned(dst)) return MXC_ERR_ALIGN;
    const int eb = (int)elem_size(dtype);
    hipStream_t st = (hipStream_t)hip_stream;
    if (src_layout == dst_layout) return launch_copy(src, dst, (size_t)n * c * h * w * eb, st);
    if (src_layout == MXC_NCHW) return launch_transpose(src, dst, n, c, h * w, eb, st);
    return launch_transpose(src, dst, n, h * w, c, eb, st);
}

const char *mxc_status_string(int status)
{
    switch (status) {
    case MXC_OK: return "ok";
    case MXC_ERR_NULL: return "a required pointer is NULL";
    case MXC_ERR_SHAPE: return "invalid shape: non-positive dimension or stride, negative pad, or empty output";
    case MXC_ERR_UNSUPPORTED: return "unsupported dtype, layout or pass";
    case MXC_ERR_WORKSPACE: return "workspace missing or too small (see mxc_conv2d_workspace_bytes)";
    case MXC_ERR_ALIGN: return "a device pointer is not 16-byte aligned";
    case MXC_ERR_LAUNCH: return "the HIP runtime rejected a kernel launch";
    default: return "unknown status";
    }
}

const char *mxc_last_variant(void) { return g_variant; }

void mxc_last_plan_key(long long *M, int *Co, int *Kd)
{
    long long m = 0;
    int co = 0, kd = 0;
    igemm_last_plan_key(&m, &co, &kd);
    if (M) *M = m;
    if (Co) *Co = co;
    if (Kd) *Kd = kd;
}

int mxc_version(void) { return 400; }

const char *mxc_tile_name(int family, int index)
{
    return family == 0 ? igemm_tile_name(index) : family == 1 ? wgrad_tile_name(index) : family == 2 ? igemm_stream_name(index) : nullptr;
}

int mxc_probe_mfma(int workgroups, int iters, void *out, size_t out_bytes, double *flops, void *hip_stream)
{
    if (!out || !flops) return MXC_ERR_NULL;
    if (workgroups <= 0 || iters <= 0) return MXC_ERR_SHAPE;
    if (out_bytes < (size_t)workgroups * 256 * sizeof(float)) return MXC_ERR_WORKSPACE;
    if (misaligned(out)) return MXC_ERR_ALIGN;
    return probe_mfma(workgroups, iters, (float *)out, flops, (hipStream_t)hip_stream);
}

}  // extern "C"
