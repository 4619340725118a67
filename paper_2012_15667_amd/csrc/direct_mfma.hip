// Direct convolution on the fp32 matrix cores (v_mfma_f32_32x32x2_f32), dataflow of Sec. 5.2.
//
// One workgroup owns an output sub-block of b images * ty rows * tx columns (npix pixels, a multiple
// of 32) by z output channels (a multiple of 32) and keeps its partial sums in accumulator registers
// for the whole channel loop; they are written to HBM once.  The contraction over (c, r, s) runs as an
// implicit GEMM:  acc[z][npix] += W[z][alpha*R*S] * X[alpha*R*S][npix], where X is never materialised:
// each lane reads its pixel's window straight out of the LDS-resident input tile xh * yh.
//
// Per stage of alpha channels the workgroup stages, with LDS-direct loads (no registers in between),
//   - the weight slab  [alpha][R*S][z]  from the re-laid-out weights wt[C][R*S][K], 16 bytes per lane;
//   - the input tile   [alpha][b][yh][xh], element-wise, padded elements fetched from a zero word.
// Two LDS buffers alternate: the loads of stage s+1 are in flight while stage s is multiplied.
//
// Wave layout: waves_m x waves_n waves; a wave owns MBW x NBW blocks of 32 x 32 partial sums.
// Inside one MFMA the two k-slices are fed by lane halves: lanes 0-31 take channel c2, lanes 32-63 take
// channel c2 + alpha/2, so that both halves use the same LDS offset per (r, s).
#include "kernels.h"

namespace iolb {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ void load_to_lds_4(const float* src, float* lds_wave_base)
{
    __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)lds_wave_base, 4, 0, 0);
}
__device__ __forceinline__ void load_to_lds_16(const float* src, float* lds_wave_base)
{
    __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)lds_wave_base, 16, 0, 0);
}

template <int MBW, int NBW, int LB>
__global__ void __launch_bounds__(LB)
direct_mfma_kernel(const float* __restrict__ x, const float* __restrict__ wt, float* __restrict__ y,
                   const float* __restrict__ zeros, DirectGeom g)
{
    extern __shared__ float lds[];
    const int tid = threadIdx.x, T = blockDim.x;
    const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // consecutive workgroup ids are dealt round-robin to the 8 XCDs; remap so that each XCD (one L2)
    // works on a contiguous range of blocks, whose channel blocks share the same input tile
    int bid = blockIdx.x;
    const int nblk = gridDim.x;
    if ((nblk & 7) == 0) bid = (bid & 7) * (nblk >> 3) + (bid >> 3);
    const int kb = bid % g.nbk; bid /= g.nbk;
    const int xb = bid % g.nbx; bid /= g.nbx;
    const int yb = bid % g.nby;
    const int nb_ = bid / g.nby;
    const int k0 = kb * g.z, x0 = xb * g.tx, y0 = yb * g.ty, n0 = nb_ * g.b;

    const int RS = g.R * g.S;
    const int HW = g.H * g.W;
    const int wfloats = g.alpha * RS * g.z;                 // weight slab, multiple of 32 floats
    const int stage_floats = (wfloats + g.alpha * g.halo + 3) & ~3;
    const int half_c = g.alpha >> 1;

    const int wm_i = wave % g.waves_m, wn_i = wave / g.waves_m;

    // per-lane read bases inside a stage buffer
    int bbase[NBW], pimg[NBW], ppy[NBW], ppx[NBW];
    const int txy = g.tx * g.ty;
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int pix = (wn_i * NBW + nb) * 32 + l32;
        pimg[nb] = pix / txy;
        const int rem = pix % txy;
        ppy[nb] = rem / g.tx;
        ppx[nb] = rem % g.tx;
        bbase[nb] = wfloats + half * half_c * g.halo + pimg[nb] * g.yh * g.xh + ppy[nb] * g.stride * g.xh +
                    ppx[nb] * g.stride;
    }
    const int abase = half * half_c * RS * g.z + wm_i * MBW * 32 + l32;

    floatx16 acc[MBW][NBW];
#pragma unroll
    for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.f;

    const int gy0 = y0 * g.stride - g.pad, gx0 = x0 * g.stride - g.pad;
    const int z4 = g.z >> 2;
    const int w_vec = g.alpha * RS * z4;                    // 16-byte elements in the weight slab
    const int yxh = g.yh * g.xh;

    auto issue_stage = [&](int c0, float* buf) {
        // weights: slab row (c, rs) holds z contiguous floats of wt
        for (int e = tid; e < w_vec; e += T) {
            const int row = e / z4, k4 = e - row * z4;
            const int ch = c0 + row / RS;
            const float* src = (ch < g.C) ? wt + ((size_t)(c0 * RS + row) * g.K + k0 + k4 * 4) : zeros;
            load_to_lds_16(src, buf + __builtin_amdgcn_readfirstlane(e - lane) * 4);
        }
        // input tile: element h of the tile for each staged channel
        for (int h = tid; h < g.halo; h += T) {
            const int im = h / yxh, r2 = h - im * yxh;
            const int hy = r2 / g.xh, hx = r2 - hy * g.xh;
            const int gy = gy0 + hy, gx = gx0 + hx;
            const bool inside = gy >= 0 && gy < g.H && gx >= 0 && gx < g.W;
            const float* src0 = x + ((size_t)(n0 + im) * g.C + c0) * HW + gy * g.W + gx;
            float* dst = buf + wfloats + __builtin_amdgcn_readfirstlane(h - lane);
            for (int c = 0; c < g.alpha; ++c) {
                const float* src = (inside && c0 + c < g.C) ? src0 + (size_t)c * HW : zeros;
                load_to_lds_4(src, dst + c * g.halo);
            }
        }
    };

    const int nstages = (g.C + g.alpha - 1) / g.alpha;
    issue_stage(0, lds);
    for (int s = 0; s < nstages; ++s) {
        __syncthreads();                                    // stage s has landed; stage s-1 is consumed
        float* cur = lds + (s & 1) * stage_floats;
        if (s + 1 < nstages) issue_stage((s + 1) * g.alpha, lds + ((s + 1) & 1) * stage_floats);

        for (int c2 = 0; c2 < half_c; ++c2) {
            const float* wrow = cur + abase + c2 * RS * g.z;
            const int xoff_c = c2 * g.halo;
            for (int r = 0; r < g.R; ++r) {
                for (int sx = 0; sx < g.S; ++sx) {
                    float a[MBW], bv[NBW];
#pragma unroll
                    for (int mb = 0; mb < MBW; ++mb) a[mb] = wrow[mb * 32];
                    const int xo = xoff_c + r * g.xh + sx;
#pragma unroll
                    for (int nb = 0; nb < NBW; ++nb) bv[nb] = cur[bbase[nb] + xo];
#pragma unroll
                    for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
                        for (int nb = 0; nb < NBW; ++nb)
                            acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mb], bv[nb], acc[mb][nb], 0, 0, 0);
                    wrow += g.z;
                }
            }
        }
    }

    // each partial sum is complete: write the block once.  Register i of a 32 x 32 block holds
    // channel 8*(i/4) + 4*half + i%4 of pixel l32.
    const size_t PQ = (size_t)g.P * g.Q;
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        float* yp = y + ((size_t)(n0 + pimg[nb]) * g.K + k0) * PQ + (size_t)(y0 + ppy[nb]) * g.Q + x0 + ppx[nb];
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb) {
            const int kbase = (wm_i * MBW + mb) * 32 + 4 * half;
#pragma unroll
            for (int i = 0; i < 16; ++i) yp[(size_t)(kbase + 8 * (i >> 2) + (i & 3)) * PQ] = acc[mb][nb][i];
        }
    }
}

// w[K][CRS] -> wt[CRS][K] through a 32 x 33 LDS tile: both sides coalesced.
__global__ void __launch_bounds__(256)
weight_relayout_kernel(const float* __restrict__ w, float* __restrict__ wt, int K, int CRS)
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
        if (c < CRS && k < K) wt[(size_t)c * K + k] = tile[tx][j];
    }
}

template <int MBW, int NBW, int LB>
hipError_t launch_one(const float* x, const float* wt, float* y, const float* zeros, const DirectGeom& g,
                      size_t shm, hipStream_t st)
{
    auto kern = direct_mfma_kernel<MBW, NBW, LB>;
    static bool raised = false;               // dynamic LDS above 64 KB needs an opt-in, once per kernel
    if (shm > 64 * 1024 && !raised) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    const int grid = g.nbk * g.nbx * g.nby * g.nbn;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(g.threads), shm, st, x, wt, y, zeros, g);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_weight_relayout(const float* w, float* wt, int K, int CRS, hipStream_t st)
{
    dim3 grid((CRS + 31) / 32, (K + 31) / 32);
    hipLaunchKernelGGL(weight_relayout_kernel, grid, dim3(256), 0, st, w, wt, K, CRS);
    return hipGetLastError();
}

hipError_t launch_direct_mfma(const float* x, const float* wt, float* y, const float* zeros,
                              const DirectGeom& g, hipStream_t st)
{
    const int npix = g.b * g.tx * g.ty;
    if (npix % 32 || g.z % 32 || (g.alpha & 1) || g.threads != 64 * g.waves_m * g.waves_n) return hipErrorInvalidValue;
    const int MB = g.z / 32, NB = npix / 32;
    if (MB % g.waves_m || NB % g.waves_n) return hipErrorInvalidValue;
    const int mbw = MB / g.waves_m, nbw = NB / g.waves_n;
    const size_t stage = ((size_t)g.alpha * ((size_t)g.R * g.S * g.z + g.halo) + 3) & ~(size_t)3;
    const size_t shm = 2 * stage * sizeof(float);
    if (shm > 160 * 1024) return hipErrorInvalidValue;
    // the register file of a compute unit holds 131072 lane-registers: a workgroup of T threads gets
    // 131072 / T per lane, of which 16 * mbw * nbw are partial sums
    if (16 * mbw * nbw + 64 > 131072 / g.threads) return hipErrorInvalidValue;
#define IOLB_CASE(M_, N_)                                                                        \
    if (mbw == M_ && nbw == N_) {                                                                \
        if (g.threads <= 256) return launch_one<M_, N_, 256>(x, wt, y, zeros, g, shm, st);       \
        if (g.threads <= 512) return launch_one<M_, N_, 512>(x, wt, y, zeros, g, shm, st);       \
        if constexpr (M_ * N_ <= 4) return launch_one<M_, N_, 1024>(x, wt, y, zeros, g, shm, st); \
    }
    IOLB_CASE(1, 1) IOLB_CASE(1, 2) IOLB_CASE(1, 3) IOLB_CASE(1, 4)
    IOLB_CASE(1, 5) IOLB_CASE(1, 6) IOLB_CASE(1, 7) IOLB_CASE(1, 8)
    IOLB_CASE(2, 1) IOLB_CASE(2, 2) IOLB_CASE(2, 3) IOLB_CASE(2, 4)
#undef IOLB_CASE
    return hipErrorInvalidValue;
}

}  // namespace iolb
