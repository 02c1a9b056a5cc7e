// Layout conversion kernels: batched 2-D transposes through LDS.
//
// NCHW -> NHWC of an activation tensor is, per image, the transpose of a
// [C][H*W] matrix; KCRS -> KRSC of a filter bank is the same with [C][R*S].
// Pure data movement: 1 read + 1 write of every element, HBM-bound.
#include "mxc_internal.h"

namespace mxc {

namespace {

constexpr int TILE = 64;

// The tile kernels run on a one-dimensional grid of batch x row tiles x column tiles workgroups (column tile
// fastest), so that neither the batch nor the row-tile count is bound by the 65535 limit of the grid's y and z.
struct TileId { unsigned bx, by, bz; };
__device__ __forceinline__ TileId tile_id(int rows, int cols)
{
    const unsigned gx = (unsigned)(cols + TILE - 1) / TILE, gy = (unsigned)(rows + TILE - 1) / TILE;
    const unsigned t = blockIdx.x / gx;
    return TileId{blockIdx.x % gx, t % gy, t / gy};
}

// One 64x64 tile per workgroup of 256 threads.  Reads are contiguous along
// `cols`, writes contiguous along `rows`; the +1 pad keeps the column reads of
// the LDS tile off a single bank.
template <typename T>
__global__ __launch_bounds__(256) void transpose_tile_kernel(const T *__restrict__ src, T *__restrict__ dst,
                                                             int rows, int cols)
{
    __shared__ T tile[TILE][TILE + 1];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const TileId id = tile_id(rows, cols);
    const int c0 = id.bx * TILE, r0 = id.by * TILE;
    const size_t base = (size_t)id.bz * rows * cols;
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

// The same transpose at vector width for 2-byte elements: 16-byte global loads and stores on both sides.
// A workgroup moves a 64 x 64 tile; a thread loads the same 8 columns of two consecutive rows, pairs the
// elements of each column into one dword (byte permutes) and writes the 8 dwords into the transposed LDS tile
// [column][row pair]; then every thread gathers 8 consecutive rows of one column (4 dwords) and stores them as
// one 16-byte chunk of the destination row.  Needs rows % 8 == 0 and cols % 8 == 0 (16-byte alignment of
// every row on both sides); ragged tile edges are handled chunk-wise.
__global__ __launch_bounds__(256) void transpose_vec16_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst,
                                                              int rows, int cols)
{
    constexpr int PITCH = 33;                              // dwords per LDS column: odd, conflict-free dword writes
    __shared__ uint32_t tile[TILE * PITCH];
    const int t = threadIdx.x;
    const TileId id = tile_id(rows, cols);
    const int c0 = id.bx * TILE, r0 = id.by * TILE;
    const size_t base = (size_t)id.bz * rows * cols;
    {
        const int cc = t & 7, rp = t >> 3;                 // 8-column chunk, row pair
        const int r = r0 + 2 * rp, c = c0 + cc * 8;
        uint4 a = make_uint4(0, 0, 0, 0), b = a;
        if (r < rows && c < cols) {                        // rows is even: r + 1 < rows as well
            a = *reinterpret_cast<const uint4 *>(src + base + (size_t)r * cols + c);
            b = *reinterpret_cast<const uint4 *>(src + base + (size_t)(r + 1) * cols + c);
        }
        const uint32_t av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // columns 2j and 2j+1: low halves and high halves of the two rows' dwords
            tile[(cc * 8 + 2 * j) * PITCH + rp] = __builtin_amdgcn_perm(bv[j], av[j], 0x05040100u);
            tile[(cc * 8 + 2 * j + 1) * PITCH + rp] = __builtin_amdgcn_perm(bv[j], av[j], 0x07060302u);
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int oc = (t >> 3) + 32 * i, q = t & 7;       // tile column, chunk of 8 rows
        const int c = c0 + oc, r = r0 + q * 8;
        if (c < cols && r < rows) {
            const uint32_t *l = tile + oc * PITCH + q * 4;
            *reinterpret_cast<uint4 *>(dst + base + (size_t)c * rows + r) = make_uint4(l[0], l[1], l[2], l[3]);
        }
    }
}

// ... and for 4-byte elements: 16-byte chunks hold 4 elements; 64 x 64 tile in four passes of 16 rows.
__global__ __launch_bounds__(256) void transpose_vec16_kernel(const uint32_t *__restrict__ src, uint32_t *__restrict__ dst,
                                                              int rows, int cols)
{
    constexpr int PITCH = 65;
    __shared__ uint32_t tile[TILE * PITCH];
    const int t = threadIdx.x;
    const TileId id = tile_id(rows, cols);
    const int c0 = id.bx * TILE, r0 = id.by * TILE;
    const size_t base = (size_t)id.bz * rows * cols;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int cc = t & 15, lr = (t >> 4) + 16 * i;
        const int r = r0 + lr, c = c0 + cc * 4;
        uint4 a = make_uint4(0, 0, 0, 0);
        if (r < rows && c < cols) a = *reinterpret_cast<const uint4 *>(src + base + (size_t)r * cols + c);
        tile[(cc * 4 + 0) * PITCH + lr] = a.x;
        tile[(cc * 4 + 1) * PITCH + lr] = a.y;
        tile[(cc * 4 + 2) * PITCH + lr] = a.z;
        tile[(cc * 4 + 3) * PITCH + lr] = a.w;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int oc = (t >> 4) + 16 * i, q = t & 15;
        const int c = c0 + oc, r = r0 + q * 4;
        if (c < cols && r < rows) {
            const uint32_t *l = tile + oc * PITCH + q * 4;
            *reinterpret_cast<uint4 *>(dst + base + (size_t)c * rows + r) = make_uint4(l[0], l[1], l[2], l[3]);
        }
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

// Same permutation for 2-byte elements, C channels, 8 pixels per thread: C 16-byte accesses on the planar side, a
// register shuffle, and C 16-byte accesses on the interleaved side.  A thread's C interleaved chunks are
// neighbours in memory (a wave-wide access of "my i-th chunk" would touch 16 bytes of every 16*C), so they pass
// through LDS and each instruction of the interleaved side covers one contiguous span of the workgroup's pixels.
// Needs pixels % 8 == 0 (keeps every access 16-byte aligned).
template <int C, bool TO_INTERLEAVED>
__global__ __launch_bounds__(256) void small_c_vec_kernel(const uint16_t *__restrict__ src, uint16_t *__restrict__ dst,
                                                          long long pixels)
{
    __shared__ uint4 chunks[256 * C];
    const int t = threadIdx.x;
    const long long blk_pix0 = (long long)blockIdx.x * 2048;           // first pixel of this workgroup
    const long long pix0 = blk_pix0 + (long long)t * 8;
    const bool mine = pix0 < pixels;
    const size_t base = (size_t)blockIdx.y * C * pixels;
    const long long blk_chunks = (min(pixels - blk_pix0, 2048ll) / 8) * C;   // 16-byte chunks of this workgroup's span
    uint16_t *inter = const_cast<uint16_t *>(TO_INTERLEAVED ? dst : src) + base + (size_t)blk_pix0 * C;
    union V { uint4 v; uint16_t e[8]; };
    V in[C], out[C];
    if (TO_INTERLEAVED) {
        if (mine) {
#pragma unroll
            for (int ch = 0; ch < C; ++ch) in[ch].v = *reinterpret_cast<const uint4 *>(src + base + (size_t)ch * pixels + pix0);
#pragma unroll
            for (int j = 0; j < 8 * C; ++j) out[j / 8].e[j % 8] = in[j % C].e[j / C];
#pragma unroll
            for (int i = 0; i < C; ++i) chunks[t * C + i] = out[i].v;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < C; ++i)
            if (i * 256 + t < blk_chunks) reinterpret_cast<uint4 *>(inter)[i * 256 + t] = chunks[i * 256 + t];
    } else {
#pragma unroll
        for (int i = 0; i < C; ++i)
            if (i * 256 + t < blk_chunks) chunks[i * 256 + t] = reinterpret_cast<const uint4 *>(inter)[i * 256 + t];
        __syncthreads();
        if (mine) {
#pragma unroll
            for (int i = 0; i < C; ++i) in[i].v = chunks[t * C + i];
#pragma unroll
            for (int j = 0; j < 8 * C; ++j) out[j % C].e[j / C] = in[j / 8].e[j % 8];
#pragma unroll
            for (int ch = 0; ch < C; ++ch) *reinterpret_cast<uint4 *>(dst + base + (size_t)ch * pixels + pix0) = out[ch].v;
        }
    }
}

template <int C>
void launch_small_c_vec(const void *src, void *dst, int batch, long long pixels, bool to_inter, hipStream_t stream)
{
    dim3 grid((unsigned)((pixels / 8 + 255) / 256), (unsigned)batch), block(256);
    if (to_inter) hipLaunchKernelGGL((small_c_vec_kernel<C, true>), grid, block, 0, stream, (const uint16_t *)src, (uint16_t *)dst, pixels);
    else hipLaunchKernelGGL((small_c_vec_kernel<C, false>), grid, block, 0, stream, (const uint16_t *)src, (uint16_t *)dst, pixels);
}

// Plain copy: every workgroup owns one contiguous span of 4 x 256 chunks of 16 bytes; a thread issues its four
// loads before the first store, so four chunks per lane are in flight.
__global__ __launch_bounds__(256) void copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16,
                                                   const unsigned char *__restrict__ tail_src,
                                                   unsigned char *__restrict__ tail_dst, int tail)
{
    typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 *s = reinterpret_cast<const u32x4 *>(src);
    u32x4 *d = reinterpret_cast<u32x4 *>(dst);
    const size_t i0 = (size_t)blockIdx.x * 1024 + threadIdx.x;
    u32x4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (i0 + 256 * j < n16) v[j] = __builtin_nontemporal_load(s + i0 + 256 * j);
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (i0 + 256 * j < n16) __builtin_nontemporal_store(v[j], d + i0 + 256 * j);
    if (blockIdx.x == 0 && (int)threadIdx.x < tail) tail_dst[threadIdx.x] = tail_src[threadIdx.x];
}

}  // namespace

bool transpose_launchable(long long batch, long long rows, long long cols)
{
    if (batch <= 0 || rows <= 0 || cols <= 0 || rows > 0x7FFFFFFFll || cols > 0x7FFFFFFFll) return false;
    const long long gx = (cols + TILE - 1) / TILE, gy = (rows + TILE - 1) / TILE;
    return gx * gy <= 0x7FFFFFFFll / batch;
}

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
    if (!transpose_launchable(batch, rows, cols)) return MXC_ERR_SHAPE;
    const long long gx = (cols + TILE - 1) / TILE, gy = (rows + TILE - 1) / TILE;
    dim3 grid((unsigned)(gx * gy * batch)), block(256);
    const int per16 = 16 / (elem_bytes > 0 ? elem_bytes : 1);
    const bool vec16 = rows % per16 == 0 && cols % per16 == 0 && ((uintptr_t)src % 16) == 0 && ((uintptr_t)dst % 16) == 0;
    if (elem_bytes == 2 && vec16)
        hipLaunchKernelGGL((void (*)(const uint16_t *, uint16_t *, int, int))transpose_vec16_kernel, grid, block, 0, stream,
                           (const uint16_t *)src, (uint16_t *)dst, rows, cols);
    else if (elem_bytes == 4 && vec16)
        hipLaunchKernelGGL((void (*)(const uint32_t *, uint32_t *, int, int))transpose_vec16_kernel, grid, block, 0, stream,
                           (const uint32_t *)src, (uint32_t *)dst, rows, cols);
    else if (elem_bytes == 2)
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
    size_t blocks = (n16 + 1023) / 1024;
    if (blocks < 1) blocks = 1;
    if (blocks > 0x7FFFFFFFull) return MXC_ERR_SHAPE;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4 *)src, (uint4 *)dst, n16,
                       (const unsigned char *)src + n16 * 16, (unsigned char *)dst + n16 * 16, tail);
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_LAUNCH;
}

}  // namespace mxc
