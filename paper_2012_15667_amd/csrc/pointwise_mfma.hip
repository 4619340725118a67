// 1 x 1 convolution (no padding) on the fp32 matrix cores: the dataflow of Sec. 5.2 for R = S = 1.
//
// Without a kernel window the pixels of an image do not interact: the H x W plane is one row of HW pixels, the
// input tile of an output sub-block is the sub-block itself (x' = x, y' = y), and the layer is, per image, the
// product  y[K][HW] = w[K][C] * x[C][HW].  An output sub-block of z channels by npix pixels keeps its partial
// sums in accumulator registers for the whole channel loop and is written once, as in the general kernel; what
// differs is the road of the inputs.  Every input element is used by exactly one wave (a wave owns all z
// channels of its pixels), so the inputs go from memory straight into the registers that feed the matrix core
// -- no LDS, no barrier on their way -- through a ring of D channel pairs per lane that is refilled as it is
// consumed: the loads run a whole stage (D steps) ahead of the multiplications; D is chosen per layer and wave
// shape so that the ring covers the latency of memory even when a SIMD has a single wave.  Only the weights are
// shared: a stage's slab of 2 D channels by z kernels goes through registers into one of two LDS buffers, read
// from the kernels as the caller holds them (w[K][C], four consecutive channels of a kernel per load) and
// transposed on the way, so that no re-layout pass runs before the kernel.
//
// A wave owns MBW x NBW blocks of 32 x 32 partial sums: z = 32 MBW channels by 32 NBW pixels.  With VEC the
// lane's NBW pixels are neighbours (pixel l32 * NBW + nb of the wave's range): one NBW-float load per channel,
// one NBW-float store per output channel; this needs HW to be a multiple of NBW.  Without it block nb holds
// pixels nb * 32 + l32 and all accesses are single floats.  As everywhere in this library the two k-slices of
// an MFMA are fed by the lane halves: lanes 0-31 take channel c, lanes 32-63 channel c + D of the stage.
// With a stride the output pixel (p, q) reads input pixel (stride p, stride q): the same kernel with the lane's
// input offsets computed from its output pixels (single-float accesses); "pixels" below are output pixels.
#include "kernels.h"
#include "lds_dma.h"

#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

namespace iolb {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a compile-time constant
template <int... I, class F>
__device__ __forceinline__ void static_for_each(std::integer_sequence<int, I...>, F&& f) { (f(std::integral_constant<int, I>{}), ...); }
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) { static_for_each(std::make_integer_sequence<int, N>{}, f); }

template <int N> struct vec_of { typedef float type __attribute__((ext_vector_type(N))); };
template <> struct vec_of<1> { typedef float type; };

// D: channel pairs per stage = depth of the input ring
template <int MBW, int NBW, int D, bool VEC>
__global__ void __launch_bounds__(256, 1)
pointwise_mfma_kernel(const float* __restrict__ x, const float* __restrict__ w, float* __restrict__ y, PointGeom g)
{
    constexpr int Z = 32 * MBW, PW_ALPHA = 2 * D;
    constexpr int SLAB = PW_ALPHA * Z;                    // floats of a stage's weights
    __shared__ float wlds[2 * SLAB];
    typedef typename vec_of<NBW>::type xvec;

    const int tid = threadIdx.x;
    const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // consecutive workgroup ids are dealt round-robin to the 8 XCDs; remap so that each XCD (one L2) works on a
    // contiguous range of blocks, in which the channel blocks of one pixel range are neighbours
    int bid = blockIdx.x;
    const int nblk = gridDim.x;
    if ((nblk & 7) == 0) bid = (bid & 7) * (nblk >> 3) + (bid >> 3);
    const int kb = bid % g.nbk;
    const int pg = bid / g.nbk;
    const int k0 = kb * Z;

    // this wave's pixel range: tile `wtile` of 32 NBW pixels of one image; waves past the last tile repeat it and
    // store nothing
    const int ntiles = g.N * g.tiles_per_image;
    int wtile = pg * g.waves + wave;
    const bool live = wtile < ntiles;
    if (!live) wtile = ntiles - 1;
    const int img = wtile / g.tiles_per_image;
    const int pbase = (wtile % g.tiles_per_image) * 32 * NBW;

    // byte offset of the lane's first pixel in channel 0 of its image, per block when the blocks are strided;
    // pixels past the image read pixel 0 of the range (always inside) and store nothing
    const unsigned HWb = 4u * (unsigned)g.HWin;                  // bytes of an input channel plane
    unsigned poff[VEC ? 1 : NBW];
    if constexpr (VEC) {                                         // stride 1: input pixel = output pixel
        const int p = pbase + l32 * NBW;
        poff[0] = 4u * (unsigned)(p < g.HW ? p : pbase);
    } else {
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            int p = pbase + nb * 32 + l32;
            if (p >= g.HW) p = pbase;
            poff[nb] = 4u * (unsigned)(g.stride == 1 ? p : (p / g.Q) * g.stride * g.Win + (p % g.Q) * g.stride);
        }
    }
    const char* ximg = reinterpret_cast<const char*>(x) + (size_t)img * g.C * HWb;    // wave-uniform

    const int nstages = (g.C + PW_ALPHA - 1) / PW_ALPHA;

    // The global loads of the channel loop are written as assembly, with explicit waits: loads complete in the
    // order they were issued, so "at most n still in flight" names exactly the load a step needs, and the order
    // below IS the pipeline -- per stage the weights first, then one input load per step behind the step's
    // MFMAs.  (Left to the compiler, the loads are gathered or sunk to their uses and every step waits for all.)
    // L: load instructions per step.
    constexpr int L = VEC ? 1 : NBW;
    constexpr int PIECES = SLAB / 4, WPT = (PIECES + 255) / 256;      // 16-byte pieces of a weight slab per thread
    constexpr int WAIT_X = (D - 1) * L + WPT < 63 ? (D - 1) * L + WPT : 63;     // issued after the inputs of a step
    constexpr int WAIT_W = D * L < 63 ? D * L : 63;                             // issued after a stage's weights

    // ring of D channel pairs: slot t holds the lane's pixels of channel 2 D s + t + D half
    typedef typename vec_of<VEC ? NBW : 1>::type xload;
    xload xr[D][L];
    auto load_inputs = [&](int s, int t) {
        int ch = s * PW_ALPHA + half * D + t;
        if (ch >= g.C) ch = g.C - 1;                      // last stage of a ragged C: read something that exists
        const unsigned coff = (unsigned)ch * HWb;
#pragma unroll
        for (int i = 0; i < L; ++i) {
            const unsigned off = coff + poff[i];
            if constexpr (VEC && NBW == 4) asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(xr[t][i]) : "v"(off), "s"(ximg));
            else if constexpr (VEC && NBW == 2) asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(xr[t][i]) : "v"(off), "s"(ximg));
            else asm volatile("global_load_dword %0, %1, %2" : "=v"(xr[t][i]) : "v"(off), "s"(ximg));
        }
    };
    // the value of pixel block nb in slot t, once the loads of the slot have landed
    auto input = [&](int t, int nb) -> float {
        if constexpr (VEC && NBW > 1) return xr[t][0][nb];
        else return xr[t][nb];
    };
    auto wait_inputs = [&](int t, auto n) {
        constexpr int N = decltype(n)::value;
        if constexpr (L == 1) wait_loads<N>(xr[t][0]);
        else if constexpr (L == 2) wait_loads<N>(xr[t][0], xr[t][1]);
        else wait_loads<N>(xr[t][0], xr[t][1], xr[t][2], xr[t][3]);
    };

    // weights of a stage: channels 2 D s .. 2 D s + 2 D - 1 of kernels k0 .. k0 + Z - 1, in 16-byte pieces (four
    // consecutive channels of one kernel: rows of w are g.Cw floats, a multiple of 4) dealt over the 256 threads --
    // with fewer pieces than threads the upper threads load a piece again and do not store it -- through registers
    // into LDS as [channel][kernel].  Kernels past K and, in the last stage, channels past the row are read from a
    // piece that exists and stored as zeros.
    constexpr int QPS = D / 2;                            // channel quads of a kernel per stage
    floatx4 wreg[WPT];
    const float* wsrc[WPT];
    bool wkernel[WPT], wlast[WPT];
    int wdst[WPT], wquad[WPT];
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
        const int piece = (tid + i * 256) % PIECES;
        const int kq = piece / QPS, cq = piece % QPS;
        wkernel[i] = k0 + kq < g.K;
        wlast[i] = (nstages - 1) * PW_ALPHA + 4 * cq < g.Cw;
        wsrc[i] = w + (size_t)(wkernel[i] ? k0 + kq : g.K - 1) * g.Cw;     // the kernel's first quad always exists
        wquad[i] = 4 * cq;
        wdst[i] = 4 * cq * Z + kq;
    }
    auto load_weights = [&](int s) {
#pragma unroll
        for (int i = 0; i < WPT; ++i) {
            const float* p = wsrc[i] + ((s + 1 < nstages || wlast[i]) ? s * PW_ALPHA + wquad[i] : 0);
            asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(wreg[i]) : "v"(p));
        }
    };
    auto store_weights = [&](float* buf, int s) {
#pragma unroll
        for (int i = 0; i < WPT; ++i) {
            wait_loads<WAIT_W>(wreg[i]);
            if (PIECES % 256 == 0 || tid + i * 256 < PIECES) {
                const bool keep = wkernel[i] && (s + 1 < nstages || wlast[i]);
#pragma unroll
                for (int j = 0; j < 4; ++j) buf[wdst[i] + j * Z] = keep ? wreg[i][j] : 0.f;
            }
        }
    };

    floatx16 acc[MBW][NBW];
#pragma unroll
    for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mb][nb][i] = 0.f;

    load_weights(0);
#pragma unroll
    for (int t = 0; t < D; ++t) load_inputs(0, t);
    store_weights(wlds, 0);
    __syncthreads();

    // One stage.  LAST: nothing is loaded any more, so a step waits for the loads of the stage's later steps only, and
    // the channels past a ragged C (read from a channel that exists) are replaced by zeros.
    auto stage = [&](int s, auto last) {
        constexpr bool LAST = decltype(last)::value;
        const float* wb = wlds + (s & 1) * SLAB + half * D * Z + l32;
        if constexpr (!LAST) load_weights(s + 1);
        float a[2][MBW];
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb) a[0][mb] = wb[mb * 32];
        static_for<D>([&](auto tc) {
            constexpr int t = decltype(tc)::value;
            if constexpr (t + 1 < D) {
#pragma unroll
                for (int mb = 0; mb < MBW; ++mb) a[(t + 1) & 1][mb] = wb[(t + 1) * Z + mb * 32];
            }
            float b[NBW];
            if constexpr (LAST) {
                wait_inputs(t, std::integral_constant<int, (D - 1 - t) * L>{});
                const bool inside = s * PW_ALPHA + half * D + t < g.C;
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) b[nb] = inside ? input(t, nb) : 0.f;
            } else {
                wait_inputs(t, std::integral_constant<int, WAIT_X>{});
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) b[nb] = input(t, nb);
            }
#pragma unroll
            for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[t & 1][mb], b[nb], acc[mb][nb], 0, 0, 0);
            if constexpr (!LAST) load_inputs(s + 1, t);
        });
        if constexpr (!LAST) {
            store_weights(wlds + ((s + 1) & 1) * SLAB, s + 1);   // the buffer last read in stage s - 1
            __syncthreads();
        }
    };
    for (int s = 0; s + 1 < nstages; ++s) stage(s, std::false_type{});
    stage(nstages - 1, std::true_type{});

    // Register i of a 32 x 32 block holds channel 8 (i / 4) + 4 half + i % 4 of the block's pixel l32.
    if (!live) return;
    const size_t HW = (size_t)g.HW;
    float* yimg = y + ((size_t)img * g.K + k0) * HW;
    if constexpr (VEC) {
        const int p = pbase + l32 * NBW;
        if (p >= g.HW) return;
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int kk = mb * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
                if (k0 + kk >= g.K) continue;
                xvec v;
                if constexpr (NBW == 1) v = acc[mb][0][i];
                else {
#pragma unroll
                    for (int nb = 0; nb < NBW; ++nb) v[nb] = acc[mb][nb][i];
                }
                // written once and not read again here: past the caches, when a lane stores 8 or 16 bytes (measured:
                // single-float nontemporal stores are up to twice as slow as plain ones)
                if constexpr (NBW > 1) __builtin_nontemporal_store(v, reinterpret_cast<xvec*>(yimg + (size_t)kk * HW + p));
                else *reinterpret_cast<xvec*>(yimg + (size_t)kk * HW + p) = v;
            }
    } else {
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            const int p = pbase + nb * 32 + l32;
            if (p >= g.HW) continue;
#pragma unroll
            for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int kk = mb * 32 + 8 * (i >> 2) + 4 * half + (i & 3);
                    if (k0 + kk < g.K) yimg[(size_t)kk * HW + p] = acc[mb][nb][i];
                }
        }
    }
}

template <int MBW, int NBW, int D>
hipError_t launch_shape(const float* x, const float* w, float* y, const PointGeom& g, hipStream_t st)
{
    const int grid = g.nbk * g.npg;
    if (g.stride == 1 && g.HW % NBW == 0)
        hipLaunchKernelGGL((pointwise_mfma_kernel<MBW, NBW, D, true>), dim3(grid), dim3(64 * g.waves), 0, st, x, w, y, g);
    else
        hipLaunchKernelGGL((pointwise_mfma_kernel<MBW, NBW, D, false>), dim3(grid), dim3(64 * g.waves), 0, st, x, w, y, g);
    return hipGetLastError();
}

// wp[k][c] = w[k][c] for c < C, 0 for C <= c < Cw
__global__ void pointwise_weight_pad_kernel(const float* __restrict__ w, float* __restrict__ wp, int K, int C, int Cw)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)K * Cw) return;
    const int k = (int)(i / Cw), c = (int)(i % Cw);
    wp[i] = c < C ? w[(size_t)k * C + c] : 0.f;
}

}  // namespace

hipError_t launch_pointwise_weight_pad(const float* w, float* wp, int K, int C, int Cw, hipStream_t st)
{
    if (K < 1 || C < 1 || Cw < C) return hipErrorInvalidValue;
    const size_t n = (size_t)K * Cw;
    hipLaunchKernelGGL(pointwise_weight_pad_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, w, wp, K, C, Cw);
    return hipGetLastError();
}

hipError_t launch_pointwise_mfma(const float* x, const float* w, float* y, const PointGeom& g, hipStream_t st)
{
    // what the kernel's indexing assumes
    if (g.N < 1 || g.C < 1 || g.HW < 1 || g.K < 1) return hipErrorInvalidValue;
    if (g.waves != 4) return hipErrorInvalidValue;
    if (g.z != 32 * g.mbw || g.Kp % g.z || g.Kp < g.K || g.nbk != g.Kp / g.z) return hipErrorInvalidValue;
    if (g.tiles_per_image != (g.HW + 32 * g.nbw - 1) / (32 * g.nbw)) return hipErrorInvalidValue;
    const long long ntiles = (long long)g.N * g.tiles_per_image;
    if (g.npg != (ntiles + g.waves - 1) / g.waves) return hipErrorInvalidValue;
    if ((long long)g.nbk * g.npg > 0x7fffffffLL) return hipErrorInvalidValue;
    // a lane's byte offset inside its image is 32 bits
    if (4LL * g.C * g.HWin >= (1LL << 32)) return hipErrorInvalidValue;
    if (g.stride < 1 || g.Q < 1 || g.HW % g.Q || g.Win < (g.Q - 1) * g.stride + 1 ||
        (long long)g.HWin < ((long long)(g.HW / g.Q - 1) * g.stride) * g.Win + (g.Q - 1) * g.stride + 1) return hipErrorInvalidValue;
    if ((reinterpret_cast<size_t>(x) | reinterpret_cast<size_t>(y) | reinterpret_cast<size_t>(w)) & 15) return hipErrorInvalidValue;
    if (g.Cw < g.C || (g.Cw & 3)) return hipErrorInvalidValue;
    // stage depths per wave shape: the fewer MFMAs a step has, the more steps cover the same time
#define IOLB_PW(M_, N_, A_) if (g.mbw == M_ && g.nbw == N_ && g.alpha == A_) return launch_shape<M_, N_, A_ / 2>(x, w, y, g, st);
    IOLB_PW(1, 1, 16) IOLB_PW(1, 1, 32)
    IOLB_PW(1, 2, 16) IOLB_PW(1, 2, 32)
    IOLB_PW(1, 4, 16) IOLB_PW(1, 4, 32)
    IOLB_PW(2, 2, 16) IOLB_PW(2, 2, 32)
    IOLB_PW(2, 4, 16) IOLB_PW(2, 4, 32)
#undef IOLB_PW
    return hipErrorInvalidValue;
}

}  // namespace iolb
