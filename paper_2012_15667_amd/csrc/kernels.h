// Internal launch interface between the C-ABI layer and the gfx950 kernels.
#ifndef IOLB_KERNELS_H
#define IOLB_KERNELS_H

#include <hip/hip_runtime.h>

#include <mutex>
#include <set>
#include <utility>

#include "iolbconv.h"

namespace iolb {

// Dynamic LDS above 64 KB needs an opt-in per kernel and device.  Done once for each pair; safe to call from
// several host threads.
inline hipError_t allow_large_lds(const void* kernel)
{
    static std::mutex guard;
    static std::set<std::pair<const void*, int>> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(guard);
    if (done.count({kernel, dev})) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess) done.insert({kernel, dev});
    return e;
}

// Geometry of one direct-convolution launch: the layer, the output sub-block b * tx * ty * z of
// Sec. 5.2 with its input tile xh * yh (x' * y' in the paper), and the block counts.
struct DirectGeom {
    int N, C, H, W, K, R, S, stride, pad, P, Q;   // pad: rows of zeros above and below
    int pad_w;                 // columns of zeros left and right (= pad except for conv_direct_pad2)
    int Kp;                    // MFMA path: K rounded up to a multiple of 32 (pitch of wt, extent of the z blocks)
    int b, tx, ty, z, alpha;
    int threads;               // workgroup size
    int waves_m, waves_n;      // MFMA path: wave grid; FMA path: channel groups, 1
    int per_thread;            // FMA path: output channels per lane
    int nbx, nby, nbn, nbk;    // blocks along W_out, H_out, batch, C_out
    int xh, yh, halo;          // input tile extents and elements per channel (b * yh * xh)
    int flat;                  // MFMA path, set by the launcher: input tile staged in flat 64-element chunks
    int w_transposed;          // weights are read with r and s exchanged: w[k][c][s'][r'] for this launch's (r', s')
    int hwc;                   // 0: x[N][C][H][W], y[N][K][P][Q];  1: x[N][H][W][C], y[N][P][Q][K]
};

// Re-layout w[K][C][R][S] -> wt[rows][Kp] (rows >= CRS = C*R*S, Kp >= K; rows beyond CRS and columns
// beyond K are zero) so that a stage's weight slab is a run of rows contiguous in K.
hipError_t launch_weight_relayout(const float* w, float* wt, int K, int Kp, int CRS, int rows, hipStream_t st);
// The same for a launch whose kernel extents (R, S) are the transposes of the stored weights' (S, R): row
// c*R*S + r*S + s of wt is taken from w[k][c][s][r].
hipError_t launch_weight_relayout_transposed(const float* w, float* wt, int K, int Kp, int C, int R, int S, int rows,
                                             hipStream_t st);

hipError_t launch_direct_fma(const float* x, const float* w, float* y, const DirectGeom& g, hipStream_t st);
// wt: re-laid-out weights with ceil(C/alpha)*alpha*R*S rows of g.Kp floats.
hipError_t launch_direct_mfma(const float* x, const float* wt, float* y, const DirectGeom& g, hipStream_t st);
// The same for the channels-innermost tensor layout (g.hwc = 1).
hipError_t launch_direct_mfma_hwc(const float* x, const float* wt, float* y, const DirectGeom& g, hipStream_t st);

// Thin layers (direct_thin.hip): 3 x 3 kernels, stride 1, C <= 4, plain NCHW tensors.  wk: K rows of
// direct_thin_row(C) floats (the 9 C elements of a kernel, zero-padded to whole 16-float pieces), 64-byte aligned,
// written from w by launch_direct_thin_rows.  Of g the layer, P, Q, pad and pad_w are used.
int direct_thin_row(int C);
hipError_t launch_direct_thin_rows(const float* w, float* wk, int K, int C, hipStream_t st);
hipError_t launch_direct_thin(const float* x, const float* wk, float* y, const DirectGeom& g, hipStream_t st);

// 1 x 1 convolution, no padding (pointwise_mfma.hip): per image y[K][HW] = w[K][C] x[C][HW] over the HW = P Q output
// pixels, whose inputs are the pixels (stride p, stride q) of the H x W planes.  A wave owns
// mbw x nbw blocks of 32 x 32 partial sums (z = 32 mbw channels by 32 nbw pixels of one image); a workgroup is
// `waves` waves on consecutive pixel ranges.  w: the kernels [K][Cw], Cw a multiple of 4 and 16-byte aligned rows
// (the caller's own w when C is a multiple of 4, else a copy with zeros in [C, Cw): launch_pointwise_weight_pad).
struct PointGeom {
    int N, C, HW, K;           // HW: output pixels per image
    int HWin, Win, Q, stride;  // input plane size and row length, output row length, stride (HWin = HW for stride 1)
    int Kp;                    // K rounded up to a multiple of z
    int Cw;                    // floats per kernel in w: C rounded up to a multiple of 4
    int z, mbw, nbw;
    int waves;                 // 4
    int alpha;                 // channels per stage: 16, 32 or 64 (twice the depth of the input ring)
    int tiles_per_image;       // ceil(HW / (32 nbw))
    int nbk;                   // Kp / z
    int npg;                   // workgroups along the pixels: ceil(N * tiles_per_image / waves)
};
hipError_t launch_pointwise_weight_pad(const float* w, float* wp, int K, int C, int Cw, hipStream_t st);
hipError_t launch_pointwise_mfma(const float* x, const float* w, float* y, const PointGeom& g, hipStream_t st);

// Winograd F(m x m, 3 x 3), unfused: kernel transform, input transform, batched product over the
// (m+2)^2 planes, output transform (steps 1-4 of Sec. 4.3).
struct WinoGeom {
    int N, C, H, W, K, m;
    int pad, P, Q;             // zero padding on every side; output extents P = H + 2 pad - 2, Q = W + 2 pad - 2
    int Cp;                    // C rounded up to whole stages: U and V carry zero rows for c in [C, Cp)
    int Kp;                    // K rounded up to a multiple of 32: U carries zero columns, M unused rows for k in [K, Kp)
    int CpU;                   // channel rows per plane of U (>= Cp; a caller-held U is padded to a multiple of 16)
    int th, tw;                // sub-domains along H_out and W_out
    int tiles;                 // N * th * tw
    int tiles_pitch;           // tiles rounded up to a whole number of blocks
    int tb, z, alpha;          // block: tb sub-domains by z channels of one plane
    int waves_m, waves_n;
};
hipError_t launch_wino_kernel_transform(const float* w, float* U, const WinoGeom& g, hipStream_t st);
hipError_t launch_wino_input_transform(const float* x, float* V, const WinoGeom& g, hipStream_t st);
hipError_t launch_wino_product(const float* U, const float* V, float* M, const WinoGeom& g, hipStream_t st);
hipError_t launch_wino_output_transform(const float* M, float* y, const WinoGeom& g, hipStream_t st);
// All four steps in one kernel, for C <= 4 with C * (m+2)^2 <= 128 (wino_fused.hip).  Its kernel-side
// factors are K rows of wino_fused_row(m, C) floats, Uk[k][xi * C + c], which launch_wino_fused_relayout
// makes from the plane-major U of launch_wino_kernel_transform.
int wino_fused_row(int m, int C);
hipError_t launch_wino_fused_relayout(const float* U, float* Uk, const WinoGeom& g, hipStream_t st);
hipError_t launch_wino_fused(const float* x, const float* Uk, float* y, const WinoGeom& g, hipStream_t st);

// All four steps in one matrix-core kernel for any channel count, m in {2, 4} (wino_fused_mfma.hip).  Its
// transformed kernels are U2[c / 2][xi][k][c % 2] with g.Cp rows (a multiple of g.alpha) and g.Kp columns (a
// multiple of g.z), written from w by launch_wino_kernel_transform_paired or re-laid out from a plane-major
// U[xi][rows][cols] by launch_wino_pair_relayout.  g.tb, g.z, g.alpha, g.waves_m, g.waves_n select the block.
hipError_t launch_wino_kernel_transform_paired(const float* w, float* U2, const WinoGeom& g, hipStream_t st);
hipError_t launch_wino_pair_relayout(const float* U, int rows, int cols, float* U2, const WinoGeom& g, hipStream_t st);
hipError_t launch_wino_fused_mfma(const float* x, const float* U2, float* y, const WinoGeom& g, hipStream_t st);
// The same with one wave per plane row and the input transform shared out over all threads (wino_fused_rows.hip).
hipError_t launch_wino_fused_rows(const float* x, const float* U2, float* y, const WinoGeom& g, hipStream_t st);

// Ceiling probes (probe.hip).  The copy moves bytes / 16 16-byte pieces; the MFMA loop runs
// PROBE_MFMA_BLOCKS workgroups of four waves, each wave PROBE_ACC MFMAs (4096 flop each) per iteration, and
// writes PROBE_MFMA_BLOCKS * 256 floats to sink.
constexpr int PROBE_COPY_BLOCKS = 8192;
constexpr int PROBE_MFMA_BLOCKS = 1024;
constexpr int PROBE_ACC = 8;
hipError_t launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
hipError_t launch_probe_mfma(float* sink, int iters, hipStream_t st);
// Waves of two kinds side by side on every SIMD: `slots` waves per SIMD, slot s playing role (roles >> 2 s) & 3;
// ticks gets PROBE_SHARE_BLOCKS * 16 clock counts (one per wave, unused ones untouched), sink one float.
constexpr int PROBE_SHARE_BLOCKS = 256;
constexpr unsigned PROBE_ROLE_MFMA = 0, PROBE_ROLE_VALU = 1;
hipError_t launch_probe_share(unsigned long long* ticks, float* sink, int slots, unsigned roles, int iters, hipStream_t st);

}  // namespace iolb

#endif
