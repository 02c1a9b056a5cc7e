// Measurement aid: the matrix-pipe ceiling of the device the library runs on.
//
// A register-resident loop of v_mfma_f32_32x32x16_bf16 with no memory traffic: every CU gets two
// workgroups of four waves (two waves per SIMD), each wave keeps four independent accumulator
// blocks in flight.  The bench times it with events and divides the known flop count by the time;
// that rate, not the datasheet's, is what a real kernel on this chip at its sustained clock can
// approach.
#include "mxc_internal.h"

namespace mxc {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PROBE_ACC = 4;          // independent accumulator blocks per wave
constexpr int PROBE_THREADS = 256;

__global__ __launch_bounds__(PROBE_THREADS) void mfma_probe_kernel(float *out, int iters)
{
    f32x16 acc[PROBE_ACC];
#pragma unroll
    for (int i = 0; i < PROBE_ACC; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(float)((threadIdx.x + e) % 7);
        b[e] = (__bf16)(float)((threadIdx.x + 3 * e) % 5);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PROBE_ACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < PROBE_ACC; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    out[(size_t)blockIdx.x * PROBE_THREADS + threadIdx.x] = s;
}

}  // namespace

int probe_mfma(int workgroups, int iters, float *out, double *flops, hipStream_t st)
{
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)workgroups), dim3(PROBE_THREADS), 0, st, out, iters);
    if (hipGetLastError() != hipSuccess) return MXC_ERR_LAUNCH;
    // per wave and iteration: PROBE_ACC instructions of 32*32*16 multiply-adds
    *flops = (double)workgroups * (PROBE_THREADS / 64) * (double)iters * PROBE_ACC * 2.0 * 32 * 32 * 16;
    return MXC_OK;
}

}  // namespace mxc
