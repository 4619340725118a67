// Winograd F(m x m, 3 x 3) convolution, m in {2, 3, 4, 6}: the four steps of Sec. 4.3 as four kernels.
//
//   step 1b  U[xi][c][k]  = (L K_{k,c} L^T)[xi]                    kernel transform (k padded to whole
//                                                                   32-channel blocks with zeros)
//   step 1a  V[xi][c][t]  = (B I_{c,t} B^T)[xi]                    input transform, t = sub-domain index
//   step 2+3 M[xi][k][t]  = sum_c U[xi][c][k] * V[xi][c][t]        element-wise product + channel sum,
//                                                                   one GEMM per transformed plane xi,
//                                                                   on the fp32 matrix cores
//   step 4   y            = A M_{k,t} A^T  (valid m x m part)      output transform
//
// xi runs over the n*n = (m+2)^2 positions of a transformed tile.  Sub-domain t = (image, tile row,
// tile column) in that order; tile (ti, tj) reads the n x n input window whose top-left corner is
// (ti*m - pad, tj*m - pad), zero outside the image (pad = 1 keeps the extents: P = H, Q = W).
//
// The transform matrices (wino_mats.h) are compile-time constants: zeros and +-1 cost nothing.
#include "kernels.h"
#include "lds_dma.h"
#include "wino_mats.h"
#include "wino_transform.h"

namespace iolb {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// step 1b: one lane per (c, k); k runs fastest so the writes of a wave are contiguous.  U has Cp rows of Kp
// columns per plane: rows [C, Cp) and columns [K, Kp) are zero.
template <int M>
__global__ void __launch_bounds__(256)
kernel_transform(const float* __restrict__ w, float* __restrict__ U, int C, int Cp, int K, int Kp)
{
    constexpr int n = Mats<M>::n;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)Cp * Kp) return;
    const int k = idx % Kp, c = idx / Kp;
    float g[3][3];
    const float* wp = w + ((size_t)k * C + c) * 9;
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int j = 0; j < 3; ++j) g[i][j] = (c < C && k < K) ? wp[i * 3 + j] : 0.f;
    float t[n][3], u[n][n];
    left_mul<M, UseL, n, 3, 3>(g, t);
    right_mul_t<M, UseL, n, 3, n>(t, u);
    const size_t plane = (size_t)Cp * Kp;
#pragma unroll
    for (int i = 0; i < n; ++i)
#pragma unroll
        for (int j = 0; j < n; ++j) U[(size_t)(i * n + j) * plane + idx] = u[i][j];
}

// step 1a: one lane per (c, t); t runs fastest.  VEC (m = 2 or 4, W a multiple of m, x aligned to
// 4m bytes): a lane loads the m columns under its own sub-domain as one aligned vector per row and takes
// the two border columns from its neighbour lanes (the sub-domains left and right of it), which replaces
// m + 2 strided 4-byte loads per row by one wide one; only the lanes at a wave boundary load their border
// column themselves.
template <int M, bool VEC>
__global__ void __launch_bounds__(256)
input_transform(const float* __restrict__ x, float* __restrict__ V, WinoGeom g)
{
    constexpr int n = Mats<M>::n;
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int c = blockIdx.y;
    if (t >= g.tiles) return;
    const int tj = t % g.tw, ti = (t / g.tw) % g.th, img = t / (g.tw * g.th);
    const int h0 = ti * M - g.pad, w0 = tj * M - g.pad;
    float d[n][n];
    if constexpr (VEC) {                                  // pad = 1 only: the own columns start at a multiple of m
        typedef float vec __attribute__((ext_vector_type(M)));
        const int lane = threadIdx.x & 63;
        const bool own_left = tj > 0 && lane == 0, own_right = tj + 1 < g.tw && lane == 63;
        // all loads first, without branches (rows outside the image or channels past C read a clamped
        // address and are zeroed afterwards), so that they are in flight together
        const int cc = c < g.C ? c : g.C - 1;
        const float* xc = x + ((size_t)img * g.C + cc) * g.H * g.W + w0 + 1;     // first own column: a multiple of m
        vec mid[n];
        float bl[n], br[n];
#pragma unroll
        for (int i = 0; i < n; ++i) {
            const int h = h0 + i, hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h);
            mid[i] = *reinterpret_cast<const vec*>(xc + (size_t)hc * g.W);
            bl[i] = br[i] = 0.f;
        }
        if (own_left) {
#pragma unroll
            for (int i = 0; i < n; ++i) {
                const int h = h0 + i, hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h);
                bl[i] = xc[(size_t)hc * g.W - 1];
            }
        }
        if (own_right) {
#pragma unroll
            for (int i = 0; i < n; ++i) {
                const int h = h0 + i, hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h);
                br[i] = xc[(size_t)hc * g.W + M];
            }
        }
#pragma unroll
        for (int i = 0; i < n; ++i) {
            const int h = h0 + i;
            const bool row = c < g.C && h >= 0 && h < g.H;
            float left = __shfl_up(mid[i][M - 1], 1), right = __shfl_down(mid[i][0], 1);
            if (own_left) left = bl[i];
            if (own_right) right = br[i];
            if (tj == 0) left = 0.f;
            if (tj + 1 == g.tw) right = 0.f;
            d[i][0] = row ? left : 0.f;
#pragma unroll
            for (int j = 0; j < M; ++j) d[i][j + 1] = row ? mid[i][j] : 0.f;
            d[i][n - 1] = row ? right : 0.f;
        }
    } else {
        // clamped addresses, zeroed afterwards: no branches, the loads of a window are in flight together
        const float* xc = x + ((size_t)img * g.C + (c < g.C ? c : g.C - 1)) * g.H * g.W;
#pragma unroll
        for (int i = 0; i < n; ++i)
#pragma unroll
            for (int j = 0; j < n; ++j) {
                const int h = h0 + i, ww = w0 + j;
                const int hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h), wc = ww < 0 ? 0 : (ww >= g.W ? g.W - 1 : ww);
                d[i][j] = xc[(size_t)hc * g.W + wc];
            }
#pragma unroll
        for (int i = 0; i < n; ++i)
#pragma unroll
            for (int j = 0; j < n; ++j) {
                const int h = h0 + i, ww = w0 + j;
                if (!(c < g.C && h >= 0 && h < g.H && ww >= 0 && ww < g.W)) d[i][j] = 0.f;
            }
    }
    float tmp[n][n], v[n][n];
    left_mul<M, UseB, n, n, n>(d, tmp);
    right_mul_t<M, UseB, n, n, n>(tmp, v);
    const size_t plane = (size_t)g.Cp * g.tiles_pitch;
    float* vp = V + (size_t)c * g.tiles_pitch + t;
#pragma unroll
    for (int i = 0; i < n; ++i)
#pragma unroll
        for (int j = 0; j < n; ++j) vp[(size_t)(i * n + j) * plane] = v[i][j];
}

// step 4: one lane per (k, t); t runs fastest.  VEC (m = 2 or 4, W a multiple of m, y aligned to 4m
// bytes): each of the m output rows of a sub-domain is one aligned vector store.
template <int M, bool VEC>
__global__ void __launch_bounds__(256)
output_transform(const float* __restrict__ Mp, float* __restrict__ y, WinoGeom g)
{
    constexpr int n = Mats<M>::n;
    const int t = blockIdx.x * 256 + threadIdx.x;
    const int k = blockIdx.y;
    if (t >= g.tiles) return;
    const int tj = t % g.tw, ti = (t / g.tw) % g.th, img = t / (g.tw * g.th);
    const size_t plane = (size_t)g.Kp * g.tiles_pitch;
    const float* mp = Mp + (size_t)k * g.tiles_pitch + t;
    float pi[n][n];
#pragma unroll
    for (int i = 0; i < n; ++i)
#pragma unroll
        for (int j = 0; j < n; ++j) pi[i][j] = mp[(size_t)(i * n + j) * plane];
    float tmp[M][n], o[M][M];
    left_mul<M, UseA, M, n, n>(pi, tmp);
    right_mul_t<M, UseA, M, n, M>(tmp, o);
    float* yp = y + ((size_t)img * g.K + k) * g.P * g.Q;
#pragma unroll
    for (int i = 0; i < M; ++i) {
        const int h = ti * M + i;
        if constexpr (VEC) {
            typedef float vec __attribute__((ext_vector_type(M)));
            vec v;
#pragma unroll
            for (int j = 0; j < M; ++j) v[j] = o[i][j];
            if (h < g.P) *reinterpret_cast<vec*>(yp + (size_t)h * g.Q + tj * M) = v;
        } else {
#pragma unroll
            for (int j = 0; j < M; ++j) {
                const int ww = tj * M + j;
                if (h < g.P && ww < g.Q) yp[(size_t)h * g.Q + ww] = o[i][j];
            }
        }
    }
}

// steps 2+3: M[xi] (K x tiles) = U[xi]^T (C x K) . V[xi] (C x tiles), one workgroup per z x tb block
// of one plane.  The block's partial sums (the temporaries of the channel summation) stay in registers
// for the whole channel loop.  Per stage, alpha rows of U (z floats) and of V (tb floats) go to LDS with
// 16-byte LDS-direct loads; two buffers alternate.  Lane halves feed the two k-slices of an MFMA with
// channels c2 and c2 + alpha/2.
template <int MBW, int NBW, int LB, bool DEEP>
__global__ void __launch_bounds__(LB, LB <= 256 ? 2 : 1)
wino_product_kernel(const float* __restrict__ U, const float* __restrict__ V, float* __restrict__ Mp, WinoGeom g)
{
    extern __shared__ float lds[];
    const int tid = threadIdx.x, T = blockDim.x;
    const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int nbk = g.Kp / g.z, nbt = g.tiles_pitch / g.tb;
    int bid = blockIdx.x;
    const int nblk = gridDim.x;
    if ((nblk & 7) == 0) bid = (bid & 7) * (nblk >> 3) + (bid >> 3);
    const int kb = bid % nbk; bid /= nbk;
    const int tbk = bid % nbt;
    const int xi = bid / nbt;
    const int k0 = kb * g.z, t0 = tbk * g.tb;
    const float* Up = U + (size_t)xi * g.CpU * g.Kp + k0;
    const float* Vp = V + (size_t)xi * g.Cp * g.tiles_pitch + t0;

    const int half_c = g.alpha >> 1;
    const int ufloats = g.alpha * g.z;
    const int stage_floats = g.alpha * (g.z + g.tb);
    const int wm_i = wave % g.waves_m, wn_i = wave / g.waves_m;
    const int abase = half * half_c * g.z + wm_i * MBW * 32 + l32;
    const int bbase = ufloats + half * half_c * g.tb + wn_i * NBW * 32 + l32;

    floatx16 acc[MBW][NBW];
#pragma unroll
    for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.f;

    const int nwaves = T >> 6;
    // rows [C, Cp) of U and V are zero, so every stage is alpha whole rows
    auto issue_stage = [&](int c0, float* buf) {
        stage_rows(Up + (size_t)c0 * g.Kp, g.Kp, g.z >> 2, g.alpha, buf, wave, nwaves, lane);
        stage_rows(Vp + (size_t)c0 * g.tiles_pitch, g.tiles_pitch, g.tb >> 2, g.alpha, buf + ufloats, wave, nwaves, lane);
    };

    const int nstages = (g.C + g.alpha - 1) / g.alpha;
    // waves w and w+4 share a SIMD: the second group stages the next buffer half a stage later than the
    // first, so that one of the two always has MFMAs to issue
    const int issue_group = (wave >> 2) & 1;
    const int issue_at = issue_group ? ((half_c >> 1) & ~1) : 0;

    auto multiply = [&](const float (&am)[MBW], const float (&bm)[NBW]) {
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb)
                acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(am[mb], bm[nb], acc[mb][nb], 0, 0, 0);
    };
    // issue order inside a step: one MFMA, then the LDS reads of the next step two at a time between the
    // following MFMAs, so that a wave never has an MFMA-free stretch
    auto interleave_step = [&]() {
        constexpr int MF = MBW * NBW, RD = MBW + NBW, PAIRS = (RD + 1) / 2;
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if constexpr (MF - 1 >= PAIRS) {
#pragma unroll
            for (int i = 0; i < PAIRS; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            }
            if constexpr (MF - 1 - PAIRS > 0) __builtin_amdgcn_sched_group_barrier(0x008, MF - 1 - PAIRS, 0);
        } else {
            __builtin_amdgcn_sched_group_barrier(0x100, RD, 0);
            if constexpr (MF > 1) __builtin_amdgcn_sched_group_barrier(0x008, MF - 1, 0);
        }
    };

    issue_stage(0, lds);
    for (int s = 0; s < nstages; ++s) {
        lds_dma_wait_all();
        __syncthreads();
        const float* cur = lds + (s & 1) * stage_floats;
        float* nxt = lds + ((s + 1) & 1) * stage_floats;
        const bool more = s + 1 < nstages;
        const int c0_next = (s + 1) * g.alpha;
        if constexpr (DEEP) {
            // alpha = 16, the usual stage depth, has instantiations of its own: the eight channel steps are
            // unrolled into one straight-line block (no loop branch, no wrap-around selects), which lets
            // the reads of step t+1 be placed between the MFMAs of step t over the whole stage
            float fa[2][MBW], fb[2][NBW];
            auto fetch = [&](int set, int t) {
                const float* ap = cur + abase + t * g.z;
                const float* bp = cur + bbase + t * g.tb;
#pragma unroll
                for (int mb = 0; mb < MBW; ++mb) fa[set][mb] = ap[mb * 32];
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) fb[set][nb] = bp[nb * 32];
            };
            fetch(0, 0);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                if (t == 0 || t == 4) {
                    if (more && issue_group == (t == 0 ? 0 : 1)) issue_stage(c0_next, nxt);
                }
                fetch((t + 1) & 1, t + 1 < 8 ? t + 1 : 0);        // after the last step: wrap, read and drop
                multiply(fa[t & 1], fb[t & 1]);
                interleave_step();
            }
        } else {
        // operands of channel step j+1 are fetched while the MFMAs of step j are issued (two register
        // sets, two steps per iteration); after the last step the fetch wraps to step 0 (read, dropped)
        const float* ap = cur + abase;
        const float* bp = cur + bbase;
        float a[MBW], bv[NBW], a1[MBW], b1[NBW];
        auto fetch = [&](float (&an)[MBW], float (&bn)[NBW], bool last) {
#pragma unroll
            for (int mb = 0; mb < MBW; ++mb) an[mb] = ap[mb * 32];
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) bn[nb] = bp[nb * 32];
            ap = last ? cur + abase : ap + g.z;
            bp = last ? cur + bbase : bp + g.tb;
        };
        fetch(a, bv, false);
#pragma unroll 1
        for (int j = 0; j < half_c; j += 2) {       // alpha is a multiple of 4: an even number of steps
            if (more && j == issue_at) issue_stage(c0_next, nxt);
            fetch(a1, b1, false);
            multiply(a, bv);
            interleave_step();
            fetch(a, bv, j + 2 >= half_c);
            multiply(a1, b1);
            interleave_step();
        }
        }
    }

    float* mp = Mp + ((size_t)xi * g.Kp + k0) * g.tiles_pitch + t0;
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int tcol = (wn_i * NBW + nb) * 32 + l32;
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb) {
            const int kbase = (wm_i * MBW + mb) * 32 + 4 * half;
#pragma unroll
            for (int i = 0; i < 16; ++i)
                mp[(size_t)(kbase + 8 * (i >> 2) + (i & 3)) * g.tiles_pitch + tcol] = acc[mb][nb][i];
        }
    }
}

template <int MBW, int NBW, int LB, bool DEEP>
hipError_t launch_product_one(const float* U, const float* V, float* Mp, const WinoGeom& g,
                              int grid, int threads, size_t shm, hipStream_t st)
{
    auto kern = wino_product_kernel<MBW, NBW, LB, DEEP>;
    if (shm > 64 * 1024) {
        const hipError_t e = allow_large_lds((const void*)kern);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(threads), shm, st, U, V, Mp, g);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_wino_kernel_transform(const float* w, float* U, const WinoGeom& g, hipStream_t st)
{
    const size_t n = (size_t)g.CpU * g.Kp;
    const int grid = (int)((n + 255) / 256);
    switch (g.m) {
    case 2: hipLaunchKernelGGL(kernel_transform<2>, dim3(grid), dim3(256), 0, st, w, U, g.C, g.CpU, g.K, g.Kp); break;
    case 3: hipLaunchKernelGGL(kernel_transform<3>, dim3(grid), dim3(256), 0, st, w, U, g.C, g.CpU, g.K, g.Kp); break;
    case 4: hipLaunchKernelGGL(kernel_transform<4>, dim3(grid), dim3(256), 0, st, w, U, g.C, g.CpU, g.K, g.Kp); break;
    case 6: hipLaunchKernelGGL(kernel_transform<6>, dim3(grid), dim3(256), 0, st, w, U, g.C, g.CpU, g.K, g.Kp); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_wino_input_transform(const float* x, float* V, const WinoGeom& g, hipStream_t st)
{
    if (g.Cp > 65535) return hipErrorInvalidValue;
    dim3 grid((g.tiles + 255) / 256, g.Cp);
    const bool vec = g.pad == 1 && g.W % g.m == 0 && (reinterpret_cast<uintptr_t>(x) & (4 * g.m - 1)) == 0;
    switch (g.m) {
    case 2:
        if (vec) hipLaunchKernelGGL((input_transform<2, true>), grid, dim3(256), 0, st, x, V, g);
        else     hipLaunchKernelGGL((input_transform<2, false>), grid, dim3(256), 0, st, x, V, g);
        break;
    case 3: hipLaunchKernelGGL((input_transform<3, false>), grid, dim3(256), 0, st, x, V, g); break;
    case 4:
        if (vec) hipLaunchKernelGGL((input_transform<4, true>), grid, dim3(256), 0, st, x, V, g);
        else     hipLaunchKernelGGL((input_transform<4, false>), grid, dim3(256), 0, st, x, V, g);
        break;
    case 6: hipLaunchKernelGGL((input_transform<6, false>), grid, dim3(256), 0, st, x, V, g); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_wino_output_transform(const float* Mp, float* y, const WinoGeom& g, hipStream_t st)
{
    if (g.K > 65535) return hipErrorInvalidValue;
    dim3 grid((g.tiles + 255) / 256, g.K);
    const bool vec = g.Q % g.m == 0 && (reinterpret_cast<uintptr_t>(y) & (4 * g.m - 1)) == 0;
    switch (g.m) {
    case 2:
        if (vec) hipLaunchKernelGGL((output_transform<2, true>), grid, dim3(256), 0, st, Mp, y, g);
        else     hipLaunchKernelGGL((output_transform<2, false>), grid, dim3(256), 0, st, Mp, y, g);
        break;
    case 3: hipLaunchKernelGGL((output_transform<3, false>), grid, dim3(256), 0, st, Mp, y, g); break;
    case 4:
        if (vec) hipLaunchKernelGGL((output_transform<4, true>), grid, dim3(256), 0, st, Mp, y, g);
        else     hipLaunchKernelGGL((output_transform<4, false>), grid, dim3(256), 0, st, Mp, y, g);
        break;
    case 6: hipLaunchKernelGGL((output_transform<6, false>), grid, dim3(256), 0, st, Mp, y, g); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_wino_product(const float* U, const float* V, float* Mp, const WinoGeom& g, hipStream_t st)
{
    if (g.tb % 32 || g.z % 32 || (g.alpha & 3) || g.Kp % g.z || g.Kp < g.K || g.tiles_pitch % g.tb || g.Cp % g.alpha || g.Cp < g.C || g.CpU < g.Cp)
        return hipErrorInvalidValue;
    const int MB = g.z / 32, NB = g.tb / 32;
    if (MB % g.waves_m || NB % g.waves_n) return hipErrorInvalidValue;
    const int mbw = MB / g.waves_m, nbw = NB / g.waves_n;
    const int threads = 64 * g.waves_m * g.waves_n;
    if (threads > 1024 || 16 * mbw * nbw + 64 > 131072 / threads) return hipErrorInvalidValue;
    const size_t shm = (g.C <= g.alpha ? 1 : 2) * sizeof(float) * (size_t)g.alpha * (g.z + g.tb);   // a single stage needs one buffer
    if (shm > 160 * 1024) return hipErrorInvalidValue;
    const int n = g.m + 2;
    const long long grid_ll = (long long)n * n * (g.Kp / g.z) * (g.tiles_pitch / g.tb);
    if (grid_ll > 0x7fffffffLL) return hipErrorInvalidValue;
    const int grid = (int)grid_ll;
    const bool deep = g.alpha == 16;                // eight channel steps per stage: the unrolled instantiations
#define IOLB_CASE(M_, N_)                                                                                      \
    if (mbw == M_ && nbw == N_) {                                                                              \
        if (threads <= 256) return deep ? launch_product_one<M_, N_, 256, true>(U, V, Mp, g, grid, threads, shm, st) : launch_product_one<M_, N_, 256, false>(U, V, Mp, g, grid, threads, shm, st); \
        if (threads <= 512) return deep ? launch_product_one<M_, N_, 512, true>(U, V, Mp, g, grid, threads, shm, st) : launch_product_one<M_, N_, 512, false>(U, V, Mp, g, grid, threads, shm, st); \
        if constexpr (M_ * N_ <= 4)                                                                            \
            return deep ? launch_product_one<M_, N_, 1024, true>(U, V, Mp, g, grid, threads, shm, st) : launch_product_one<M_, N_, 1024, false>(U, V, Mp, g, grid, threads, shm, st);               \
    }
    IOLB_CASE(1, 1) IOLB_CASE(1, 2) IOLB_CASE(1, 3) IOLB_CASE(1, 4)
    IOLB_CASE(1, 5) IOLB_CASE(1, 6) IOLB_CASE(1, 7) IOLB_CASE(1, 8)
    IOLB_CASE(2, 1) IOLB_CASE(2, 2) IOLB_CASE(2, 3) IOLB_CASE(2, 4)
#undef IOLB_CASE
    return hipErrorInvalidValue;
}

}  // namespace iolb
