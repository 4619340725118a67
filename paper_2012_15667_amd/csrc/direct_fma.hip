// Direct convolution, plain fp32 FMA path (Sec. 5.2 dataflow): the fallback for layers on which no matrix-core
// tile fits the LDS or none covers 64 pixels (very large kernels: an 11 x 11 stride-4 first layer), and for
// callers that ask for an FMA tile.
//
// One workgroup owns an output sub-block of b images * ty rows * tx columns * z channels and keeps
// its partial sums in registers for the whole channel loop.  Each stage copies alpha channels of the
// input tile xh * yh (zero-filled outside the image) and the matching weight slab into LDS, then
// every lane updates its pixel for `per_thread` output channels.  Outputs are written once.
// Both tensor layouts (channels outermost or innermost, g.hwc) share the kernel; the weights are
// w[K][C][R][S] in either case.
#include "kernels.h"

namespace iolb {

namespace {

template <int ZT>
__global__ void __launch_bounds__(256)
direct_fma_kernel(const float* __restrict__ x, const float* __restrict__ w, float* __restrict__ y, DirectGeom g)
{
    extern __shared__ float lds[];
    const int tid = threadIdx.x, T = blockDim.x;
    int t = blockIdx.x;
    const int kb = t % g.nbk; t /= g.nbk;
    const int xb = t % g.nbx; t /= g.nbx;
    const int yb = t % g.nby;
    const int nb = t / g.nby;
    const int k0 = kb * g.z, x0 = xb * g.tx, y0 = yb * g.ty, n0 = nb * g.b;

    const int RS = g.R * g.S;
    const int npix = g.b * g.tx * g.ty;
    const int lanes = T / g.waves_m;              // pixel lanes; waves_m holds the channel groups
    const int lp = tid % lanes, kg = tid / lanes;
    const bool active = lp < npix;
    const int img = lp / (g.tx * g.ty);
    const int py = (lp % (g.tx * g.ty)) / g.tx, px = lp % g.tx;
    const int pix_off = img * g.yh * g.xh + py * g.stride * g.xh + px * g.stride;

    float* xs = lds;                              // [alpha][halo]
    float* ws = lds + g.alpha * g.halo;           // [alpha][RS][z]
    float acc[ZT];
#pragma unroll
    for (int j = 0; j < ZT; ++j) acc[j] = 0.f;

    const int gy0 = y0 * g.stride - g.pad, gx0 = x0 * g.stride - g.pad_w;
    for (int c0 = 0; c0 < g.C; c0 += g.alpha) {
        __syncthreads();
        for (int i = tid; i < g.alpha * g.halo; i += T) {
            const int c = i / g.halo, h = i % g.halo;
            const int im = h / (g.yh * g.xh), hy = (h % (g.yh * g.xh)) / g.xh, hx = h % g.xh;
            const int gy = gy0 + hy, gx = gx0 + hx;
            float v = 0.f;
            if (c0 + c < g.C && gy >= 0 && gy < g.H && gx >= 0 && gx < g.W)
                v = g.hwc ? x[(((size_t)(n0 + im) * g.H + gy) * g.W + gx) * g.C + c0 + c]
                          : x[(((size_t)(n0 + im) * g.C + c0 + c) * g.H + gy) * g.W + gx];
            xs[i] = v;
        }
        for (int i = tid; i < g.alpha * RS * g.z; i += T) {
            const int kk = i / (g.alpha * RS), crs = i % (g.alpha * RS);       // crs fastest: contiguous reads
            const int c = crs / RS, rs = crs % RS;
            float v = 0.f;
            // w_transposed: this launch's (r, s) is stored as w[k][c][s][r] (stored extents S x R)
            const int src = g.w_transposed ? (rs % g.S) * g.R + rs / g.S : rs;
            if (c0 + c < g.C) v = w[((size_t)(k0 + kk) * g.C + c0 + c) * RS + src];
            ws[crs * g.z + kk] = v;
        }
        __syncthreads();
        if (active) {
            for (int c = 0; c < g.alpha; ++c)
                for (int r = 0; r < g.R; ++r)
                    for (int s = 0; s < g.S; ++s) {
                        const float xv = xs[c * g.halo + pix_off + r * g.xh + s];
                        const float* wp = ws + ((c * RS + r * g.S + s) * g.z + kg * g.per_thread);
#pragma unroll
                        for (int j = 0; j < ZT; ++j)
                            if (j < g.per_thread) acc[j] = __builtin_fmaf(xv, wp[j], acc[j]);
                    }
        }
    }
    if (active) {
#pragma unroll
        for (int j = 0; j < ZT; ++j) {
            if (j < g.per_thread) {
                const int k = k0 + kg * g.per_thread + j;
                if (g.hwc) y[(((size_t)(n0 + img) * g.P + y0 + py) * g.Q + x0 + px) * g.K + k] = acc[j];
                else       y[(((size_t)(n0 + img) * g.K + k) * g.P + y0 + py) * g.Q + x0 + px] = acc[j];
            }
        }
    }
}

}  // namespace

hipError_t launch_direct_fma(const float* x, const float* w, float* y, const DirectGeom& g, hipStream_t st)
{
    const int grid = g.nbk * g.nbx * g.nby * g.nbn;
    const size_t shm = sizeof(float) * (size_t)g.alpha * ((size_t)g.halo + (size_t)g.R * g.S * g.z);
    if (g.threads < 64 || g.threads > 256 || g.per_thread < 1 || g.per_thread > 16 || shm > 160 * 1024)
        return hipErrorInvalidValue;
    auto launch = [&](auto kern) {
        hipLaunchKernelGGL(kern, dim3(grid), dim3(g.threads), shm, st, x, w, y, g);
        return hipGetLastError();
    };
    hipError_t e = hipSuccess;
    if (shm > 64 * 1024) {
        // opt in to more than the default dynamic LDS once per instantiation
        e = hipFuncSetAttribute((const void*)direct_fma_kernel<16>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        return launch(direct_fma_kernel<16>);
    }
    if (g.per_thread <= 1) return launch(direct_fma_kernel<1>);
    if (g.per_thread <= 2) return launch(direct_fma_kernel<2>);
    if (g.per_thread <= 4) return launch(direct_fma_kernel<4>);
    if (g.per_thread <= 8) return launch(direct_fma_kernel<8>);
    return launch(direct_fma_kernel<16>);
}

}  // namespace iolb
