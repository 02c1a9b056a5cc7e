// The weight update that consumes the fp32 gradient of mxc_conv2d_bwd_weight:
//     v' = momentum*v - lr*(g + wd*w),   w' = w + v'
// on fp32 master weights, with an optional bf16 copy of w' for the next forward pass (rounded to
// nearest even from the fp32 result).  Elementwise and HBM-bound: 12 bytes read and 8 (+2) bytes
// written per weight; four weights per thread, 16-byte accesses.
#include "mxc_internal.h"

namespace mxc {
namespace {

__device__ __forceinline__ float step_one(float w, float g, float &v, float lr, float momentum, float wd)
{
    v = momentum * v - lr * (g + wd * w);
    return w + v;
}

template <bool HAS_V, bool HAS_COPY>
__global__ __launch_bounds__(256) void sgd_update_kernel(float *__restrict__ w, const float *__restrict__ g, float *__restrict__ v,
                                                         bf16_t *__restrict__ w_copy, size_t n, float lr, float momentum, float wd)
{
    const size_t i4 = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
    if (i4 >= n) return;
    if (i4 + 4 <= n) {
        float4 ww = *reinterpret_cast<const float4 *>(w + i4);
        const float4 gg = *reinterpret_cast<const float4 *>(g + i4);
        float4 vv = HAS_V ? *reinterpret_cast<const float4 *>(v + i4) : make_float4(0.f, 0.f, 0.f, 0.f);
        ww.x = step_one(ww.x, gg.x, vv.x, lr, momentum, wd);
        ww.y = step_one(ww.y, gg.y, vv.y, lr, momentum, wd);
        ww.z = step_one(ww.z, gg.z, vv.z, lr, momentum, wd);
        ww.w = step_one(ww.w, gg.w, vv.w, lr, momentum, wd);
        *reinterpret_cast<float4 *>(w + i4) = ww;
        if (HAS_V) *reinterpret_cast<float4 *>(v + i4) = vv;
        if (HAS_COPY) {
            const uint2 c = make_uint2((uint32_t)f32_to_bf16(ww.x) | ((uint32_t)f32_to_bf16(ww.y) << 16),
                                       (uint32_t)f32_to_bf16(ww.z) | ((uint32_t)f32_to_bf16(ww.w) << 16));
            *reinterpret_cast<uint2 *>(w_copy + i4) = c;
        }
        return;
    }
    for (size_t i = i4; i < n; ++i) {
        float vv = HAS_V ? v[i] : 0.f;
        const float ww = step_one(w[i], g[i], vv, lr, momentum, wd);
        w[i] = ww;
        if (HAS_V) v[i] = vv;
        if (HAS_COPY) w_copy[i] = f32_to_bf16(ww);
    }
}

}  // namespace

int sgd_update(size_t n, float *w, const float *g, float *v, void *w_copy, float lr, float momentum, float wd, hipStream_t st)
{
    const size_t blocks = (n + 1023) / 1024;
    if (blocks > 0x7FFFFFFFull) return MXC_ERR_SHAPE;
    const dim3 grid((unsigned)blocks), block(256);
    bf16_t *c = (bf16_t *)w_copy;
    if (v && c) hipLaunchKernelGGL((sgd_update_kernel<true, true>), grid, block, 0, st, w, g, v, c, n, lr, momentum, wd);
    else if (v) hipLaunchKernelGGL((sgd_update_kernel<true, false>), grid, block, 0, st, w, g, v, c, n, lr, momentum, wd);
    else if (c) hipLaunchKernelGGL((sgd_update_kernel<false, true>), grid, block, 0, st, w, g, v, c, n, lr, momentum, wd);
    else hipLaunchKernelGGL((sgd_update_kernel<false, false>), grid, block, 0, st, w, g, v, c, n, lr, momentum, wd);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

}  // namespace mxc
