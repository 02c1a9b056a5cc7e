// Layout conversion kernels: batched 2-D transposes through LDS.
//
// NCHW -> NHWC of an activation tensor is, per image, the transpose of a
// [C][H*W] matrix; KCRS -> KRSC of a filter bank is the same with [C][R*S].
// Pure data movement: 1 read + 1 write of every element, HBM-bound.
#include "mxc_internal.h"

namespace mxc {

namespace {

constexpr int TILE = 64;

// One 64x64 tile per workgroup of 256 threads.  Reads are contiguous along
// `cols`, writes contiguous along `rows`; the +1 pad keeps the column reads of
// the LDS tile off a single bank.
template <typename T>
__global__ __launch_bounds__(256) void transpose_tile_kernel(const T *__restrict__ src, T *__restrict__ dst,
                                                             int rows, int cols)
{
    __shared__ T tile[TILE][TILE + 1];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int c0 = blockIdx.x * TILE, r0 = blockIdx.y * TILE;
    const size_t base = (size_t)blockIdx.z * rows * cols;
#pragma unroll
    for (int i = 0; i < TILE; i += 4) {
        const int r = r0 + ty + i, c = c0 + tx;
        if (r < rows && c < cols) tile[ty + i][tx] = src[base + (size_t)r * cols + c];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < TILE; i += 4) {
        const int c = c0 + ty + i, r = r0 + tx;
        if (r < rows && c < cols) dst[base + (size_t)c * rows + r] = tile[tx][ty + i];
    }
}

// Few channels (c <= 8): one thread per pixel.  planar[b][c][pixels] <-> interleaved[b][pixels][c];
// both sides are contiguous across the lanes of a wave.
template <typename T, bool TO_INTERLEAVED>
__global__ __launch_bounds__(256) void small_c_kernel(const T *__restrict__ src, T *__restrict__ dst, int c, long long pixels)
{
    const long long pix = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (pix >= pixels) return;
    const size_t base = (size_t)blockIdx.y * c * pixels;
    for (int ch = 0; ch < c; ++ch) {
        if (TO_INTERLEAVED) dst[base + (size_t)pix * c + ch] = src[base + (size_t)ch * pixels + pix];
        else dst[base + (size_t)ch * pixels + pix] = src[base + (size_t)pix * c + ch];
    }
}

// Same permutation for 2-byte elements, C channels, 8 pixels per thread: C 16-byte loads, a register
// shuffle, C 16-byte stores.  Needs pixels % 8 == 0 (keeps every access 16-byte aligned).
template <int C, bool TO_INTERLEAVED>
__global__ __launch_bounds__(256) void small_c_vec_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst,
                                                          long long pixels)
{
    const long long pix0 = ((long long)blockIdx.x * blockDim.x + threadIdx.x) * 8;
    if (pix0 >= pixels) return;
    const size_t base = (size_t)blockIdx.y * C * pixels;
    union V { uint4 v; uint16_t e[8]; };
    V in[C], out[C];
    if (TO_INTERLEAVED) {
#pragma unroll
        for (int ch = 0; ch < C; ++ch) in[ch].v = *reinterpret_cast<const uint4 *>(src + base + (size_t)ch * pixels + pix0);
#pragma unroll
        for (int j = 0; j < 8 * C; ++j) out[j / 8].e[j % 8] = in[j % C].e[j / C];
#pragma unroll
        for (int i = 0; i < C; ++i) *reinterpret_cast<uint4 *>(dst + base + (size_t)pix0 * C + i * 8) = out[i].v;
    } else {
#pragma unroll
        for (int i = 0; i < C; ++i) in[i].v = *reinterpret_cast<const uint4 *>(src + base + (size_t)pix0 * C + i * 8);
#pragma unroll
        for (int j = 0; j < 8 * C; ++j) out[j % C].e[j / C] = in[j / 8].e[j % 8];
#pragma unroll
        for (int ch = 0; ch < C; ++ch) *reinterpret_cast<uint4 *>(dst + base + (size_t)ch * pixels + pix0) = out[ch].v;
    }
}

template <int C>
void launch_small_c_vec(const void *src, void *dst, int batch, long long pixels, bool to_inter, hipStream_t stream)
{
    dim3 grid((unsigned)((pixels / 8 + 255) / 256), (unsigned)batch), block(256);
    if (to_inter) hipLaunchKernelGGL((small_c_vec_kernel<C, true>), grid, block, 0, stream, (const uint16_t *)src, (uint16_t *)dst, pixels);
    else hipLaunchKernelGGL((small_c_vec_kernel<C, false>), grid, block, 0, stream, (const uint16_t *)src, (uint16_t *)dst, pixels);
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16,
                                                   const unsigned char *__restrict__ tail_src,
                                                   unsigned char *__restrict__ tail_dst, int tail)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
    if (blockIdx.x == 0 && (int)threadIdx.x < tail) tail_dst[threadIdx.x] = tail_src[threadIdx.x];
}

}  // namespace

int launch_transpose(const void *src, void *dst, int batch, int rows, int cols, int elem_bytes, hipStream_t stream)
{
    if (batch <= 0 || rows <= 0 || cols <= 0) return MXC_ERR_SHAPE;
    if ((rows <= 8 || cols <= 8) && batch <= 65535 && (elem_bytes == 2 || elem_bytes == 4)) {
        const bool to_inter = rows <= 8;           // [c][pixels] -> [pixels][c]
        const int c = to_inter ? rows : cols;
        const long long pixels = to_inter ? cols : rows;
        if (elem_bytes == 2 && pixels % 8 == 0 && c >= 2 && c <= 4) {
            if (c == 2) launch_small_c_vec<2>(src, dst, batch, pixels, to_inter, stream);
            else if (c == 3) launch_small_c_vec<3>(src, dst, batch, pixels, to_inter, stream);
            else launch_small_c_vec<4>(src, dst, batch, pixels, to_inter, stream);
            return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
        }
        dim3 grid((unsigned)((pixels + 255) / 256), (unsigned)batch), block(256);
        if (elem_bytes == 2) {
            if (to_inter) hipLaunchKernelGGL((small_c_kernel<uint16_t, true>), grid, block, 0, stream, (const uint16_t *)src, (uint16_t *)dst, c, pixels);
            else hipLaunchKernelGGL((small_c_kernel<uint16_t, false>), grid, block, 0, stream, (const uint16_t *)src, (uint16_t *)dst, c, pixels);
        } else {
            if (to_inter) hipLaunchKernelGGL((small_c_kernel<uint32_t, true>), grid, block, 0, stream, (const uint32_t *)src, (uint32_t *)dst, c, pixels);
            else hipLaunchKernelGGL((small_c_kernel<uint32_t, false>), grid, block, 0, stream, (const uint32_t *)src, (uint32_t *)dst, c, pixels);
        }
        return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
    }
    const unsigned gx = (unsigned)((cols + TILE - 1) / TILE), gy = (unsigned)((rows + TILE - 1) / TILE);
    if (gy > 65535u || (unsigned)batch > 65535u) return MXC_ERR_SHAPE;
    dim3 grid(gx, gy, (unsigned)batch), block(256);
    if (elem_bytes == 2)
        hipLaunchKernelGGL(transpose_tile_kernel<uint16_t>, grid, block, 0, stream, (const uint16_t *)src,
                           (uint16_t *)dst, rows, cols);
    else if (elem_bytes == 4)
        hipLaunchKernelGGL(transpose_tile_kernel<uint32_t>, grid, block, 0, stream, (const uint32_t *)src,
                           (uint32_t *)dst, rows, cols);
    else
        return MXC_ERR_UNSUPPORTED;
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

int launch_copy(const void *src, void *dst, size_t bytes, hipStream_t stream)
{
    if (bytes == 0) return MXC_OK;
    const size_t n16 = bytes / 16;
    const int tail = (int)(bytes % 16);
    size_t blocks = (n16 + 255) / 256;
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4 *)src, (uint4 *)dst, n16,
                       (const unsigned char *)src + n16 * 16, (unsigned char *)dst + n16 * 16, tail);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

}  // namespace mxc
