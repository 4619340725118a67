// Ceiling probes: what this device delivers on the two resources that bound the convolution kernels -- a
// streaming copy (HBM) and a loop of independent fp32 MFMAs with operands held in registers (matrix cores).
// Roofline fractions can then be quoted against measured as well as published peaks.
#include <hip/hip_runtime.h>

#include "kernels.h"

namespace iolb {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

__global__ void __launch_bounds__(256)
probe_copy_kernel(const floatx4* __restrict__ src, floatx4* __restrict__ dst, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

// Every wave keeps PROBE_ACC independent 32 x 32 accumulator blocks and issues `iters` rounds of one
// v_mfma_f32_32x32x2_f32 per block: no memory traffic inside the loop.
__global__ void __launch_bounds__(256)
probe_mfma_kernel(float* __restrict__ sink, int iters)
{
    floatx16 acc[PROBE_ACC];
#pragma unroll
    for (int i = 0; i < PROBE_ACC; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
    const float a = 1.f + (float)(threadIdx.x & 7), b = 0.5f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PROBE_ACC; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < PROBE_ACC; ++i)
#pragma unroll
        for (int j = 0; j < 16; ++j) s += acc[i][j];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// How the waves of one SIMD share its fp32 pipeline.  A workgroup has 4 * slots waves, so every SIMD gets `slots`
// of them; the waves of slot s (waves 4 s .. 4 s + 3) all play role (roles >> 2 s) & 3:
//   PROBE_ROLE_MFMA  iters rounds of 8 v_mfma_f32_32x32x2_f32 on four accumulators (512 matrix cycles per round);
//   PROBE_ROLE_VALU  iters rounds of 64 v_fma_f32 on four dependent chains.
// Each wave writes the clock ticks it took (s_memtime around its loop) to ticks[block * 16 + wave].
__global__ void __launch_bounds__(1024)
probe_share_kernel(unsigned long long* __restrict__ ticks, float* __restrict__ sink, unsigned roles, int iters)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const unsigned role = (roles >> (2 * (wave >> 2))) & 3u;
    floatx16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
    const float a = lane * 0.001f, b = 1.0f, c1 = 0.5f;
    float v[4] = {1.f, 2.f, 3.f, 4.f};
    __syncthreads();
    const unsigned long long t0 = __builtin_amdgcn_s_memtime();
    if (role == PROBE_ROLE_MFMA) {
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j & 3] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[j & 3], 0, 0, 0);
        }
    } else if (role == PROBE_ROLE_VALU) {
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int j = 0; j < 64; ++j) asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(v[j & 3]) : "v"(c1));
        }
    }
    const unsigned long long t1 = __builtin_amdgcn_s_memtime();
    if (lane == 0) ticks[(size_t)blockIdx.x * 16 + wave] = t1 - t0;
    float s = v[0] + v[1] + v[2] + v[3];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i];
    if (s == 123.456f) sink[0] = s;                       // keeps the loops alive; never true
}

}  // namespace

hipError_t launch_probe_share(unsigned long long* ticks, float* sink, int slots, unsigned roles, int iters, hipStream_t st)
{
    if (slots < 1 || slots > 4) return hipErrorInvalidValue;
    hipLaunchKernelGGL(probe_share_kernel, dim3(PROBE_SHARE_BLOCKS), dim3(256 * slots), 0, st, ticks, sink, roles, iters);
    return hipGetLastError();
}

hipError_t launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t st)
{
    hipLaunchKernelGGL(probe_copy_kernel, dim3(PROBE_COPY_BLOCKS), dim3(256), 0, st,
                       static_cast<const floatx4*>(src), static_cast<floatx4*>(dst), bytes / 16);
    return hipGetLastError();
}

hipError_t launch_probe_mfma(float* sink, int iters, hipStream_t st)
{
    hipLaunchKernelGGL(probe_mfma_kernel, dim3(PROBE_MFMA_BLOCKS), dim3(256), 0, st, sink, iters);
    return hipGetLastError();
}

}  // namespace iolb
