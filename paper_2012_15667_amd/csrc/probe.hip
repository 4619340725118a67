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

}  // namespace

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
