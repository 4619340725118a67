// Direct convolution on the matrix cores, x[N][C][H][W] -> y[N][K][P][Q] instantiations, and the
// weight re-layout pre-passes shared by all tensor layouts.
#include "direct_mfma_impl.h"

namespace iolb {

namespace {

// w[K][CRS] -> wt[rows][Kp] through a 32 x 33 LDS tile: both sides coalesced.  rows >= CRS, Kp >= K; the
// rows beyond CRS (channels added to fill the last stage) and the columns beyond K are written as zeros.
__global__ void __launch_bounds__(256)
weight_relayout_kernel(const float* __restrict__ w, float* __restrict__ wt, int K, int Kp, int CRS, int rows)
{
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;      // 32 x 8
    const int c0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
    for (int j = ty; j < 32; j += 8) {
        const int k = k0 + j, c = c0 + tx;
        tile[j][tx] = (k < K && c < CRS) ? w[(size_t)k * CRS + c] : 0.f;
    }
    __syncthreads();
    for (int j = ty; j < 32; j += 8) {
        const int c = c0 + j, k = k0 + tx;
        if (c < rows && k < Kp) wt[(size_t)c * Kp + k] = tile[tx][j];
    }
}

// The transposed-kernel variant: row (c, r, s) of wt comes from w[k][c][s][r] (stored extents S x R).  A few
// hundred kilobytes at most: one lane per element of wt, writes coalesced along k.
__global__ void __launch_bounds__(256)
weight_relayout_transposed_kernel(const float* __restrict__ w, float* __restrict__ wt, int K, int Kp, int C, int R, int S,
                                  int rows)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)rows * Kp) return;
    const int k = idx % Kp, row = idx / Kp;
    const int RS = R * S, c = row / RS, rs = row % RS, r = rs / S, s_ = rs % S;
    wt[idx] = (k < K && c < C) ? w[((size_t)k * C + c) * RS + s_ * R + r] : 0.f;
}

}  // namespace

hipError_t launch_weight_relayout_transposed(const float* w, float* wt, int K, int Kp, int C, int R, int S, int rows,
                                             hipStream_t st)
{
    const size_t n = (size_t)rows * Kp;
    hipLaunchKernelGGL(weight_relayout_transposed_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, w, wt, K, Kp,
                       C, R, S, rows);
    return hipGetLastError();
}

hipError_t launch_weight_relayout(const float* w, float* wt, int K, int Kp, int CRS, int rows, hipStream_t st)
{
    dim3 grid((rows + 31) / 32, (Kp + 31) / 32);
    hipLaunchKernelGGL(weight_relayout_kernel, grid, dim3(256), 0, st, w, wt, K, Kp, CRS, rows);
    return hipGetLastError();
}

hipError_t launch_direct_mfma(const float* x, const float* wt, float* y, const DirectGeom& g, hipStream_t st)
{
    return launch_direct_mfma_layout<false>(x, wt, y, g, st);
}

}  // namespace iolb
