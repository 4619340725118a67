// Winograd F(m x m, 3 x 3) for layers with many channels: the fused dataflow of Sec. 5.3 on the fp32 matrix
// cores.  One workgroup owns a block of tb sub-domains by z output channels and keeps ALL (m+2)^2 planes of its
// channel-summation temporaries (the Pi of step 3, Sec. 4.3) in accumulator registers for the whole channel
// loop; the transformed inputs (step 1) are made inside the workgroup, per stage of ALPHA channels, straight
// into the LDS buffer the products read, and the output transform (step 4) is applied to the accumulators.
// Neither the transformed inputs nor the temporaries ever reach memory: the layer reads x and the transformed
// kernels and writes y.
//
// Wave layout.  A 32 x 32 block (32 sub-domains by 32 channels) of one plane is one v_mfma_f32_32x32x2_f32
// accumulator of 16 registers.  A wave owns one ROW of m+2 planes of one 32 x 32 block, so a compute unit
// runs (m+2) * blocks light waves (16 for F(2x2) with 2 x 2 blocks).  What they can hide for each other is memory
// and LDS latency, not arithmetic: plain VALU instructions and fp32 MFMAs share one pipeline per SIMD, and a wave
// that streams MFMAs keeps the VALU instructions of the SIMD's other waves waiting, so every vector instruction
// of the transforms is paid in matrix time and the transform is kept to its additions.
//
// This file holds the variant in which a LANE transforms a whole window (used for m = 2, whose 4 x 4 windows
// are small; wino_fused_rows.hip shares the transform out differently for m = 4).  Per stage the workgroup
//   - loads the (m+2) x (m+2) input windows of its sub-domains from global memory into registers (buffer loads
//     issued one stage ahead, elements outside the image zero-filled by the hardware's range check; one lane per
//     (sub-domain, channel), the waves 0 .. ALPHA-1 take one channel each), transforms them (B d B^T) and writes
//     them to LDS as V[channel pair][plane][sub-domain][2];
//   - copies the stage's slab of the transformed kernels, U2[channel pair][plane][k][2], to LDS with LDS-direct
//     loads (issued one stage ahead: one by every wave, the rest by the waves without a transform task);
//   - multiplies: per plane and group of four channels one 8-byte LDS read per operand feeds two MFMAs (lane
//     halves take channel pairs 2j and 2j + 1, so both halves use the same offsets).
// Two LDS buffers alternate; one barrier per stage.  The output transform  Y = A Pi A^T  is split around an
// exchange through LDS: wave i applies A^T from the right to its row, T[i][b] = sum_j Pi[i][j] A[b][j]; the wave
// that finishes register r then reads the (m+2) x m values of its lanes, applies A from the left and stores.
#include "kernels.h"
#include "lds_dma.h"
#include "wino_mats.h"
#include "wino_transform.h"

namespace iolb {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// U2[cp][xi][k][2] = (L g_{k, 2 cp + e} L^T)[xi], e = 0, 1: the transformed kernels in the channel-pair-major
// layout whose stage slabs are contiguous runs.  One lane per (c, k), k fastest.  Rows [C, Cp) and columns
// [K, Kp) are zero.
template <int M>
__global__ void __launch_bounds__(256)
kernel_transform_paired(const float* __restrict__ w, float* __restrict__ U2, int C, int Cp, int K, int Kp)
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
    float* up = U2 + (((size_t)(c >> 1) * n * n) * Kp + k) * 2 + (c & 1);
#pragma unroll
    for (int i = 0; i < n; ++i)
#pragma unroll
        for (int j = 0; j < n; ++j) up[(size_t)(i * n + j) * Kp * 2] = u[i][j];
}

// U2[cp][xi][k][e] = U[xi][2 cp + e][k] for a plane-major U with `rows` channel rows and `cols` columns; zero
// where U has no entry.
__global__ void __launch_bounds__(256)
pair_relayout_kernel(const float* __restrict__ U, int rows, int cols, float* __restrict__ U2, int Cp, int Kp, int planes)
{
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)planes * Cp * Kp) return;
    const int e = idx & 1;
    const size_t q = idx >> 1;
    const int k = q % Kp;
    const int xi = (q / Kp) % planes, cp = q / ((size_t)Kp * planes);
    const int c = 2 * cp + e;
    U2[idx] = (c < rows && k < cols) ? U[((size_t)xi * rows + c) * cols + k] : 0.f;
}

// out[ROWS] = Mx[ROWS][IN] * in[IN], Mx = Sel's matrix of Mats<M>, coefficients folded at compile time.
template <int M, class Sel, int ROWS, int IN>
__device__ __forceinline__ void mat_vec(const float (&in)[IN], float (&out)[ROWS])
{
    static_for<ROWS>([&](auto i) {
        float s = 0.f;
        bool first = true;
        static_for<IN>([&](auto k) { accumulate<M, Sel, decltype(i)::value, decltype(k)::value>(s, first, in[k]); });
        out[decltype(i)::value] = s;
    });
}

// M: output tile edge.  WT x WK: 32 x 32 blocks of the workgroup along sub-domains and channels (tb = 32 WT,
// z = 32 WK).  ALPHA: channels per stage, one transform wave each.
// VEC (pad = 1, W a multiple of M, x aligned to 4 M bytes): a lane loads the M columns under its own
// sub-domain as one aligned vector per window row and the two border columns as single floats, which replaces
// (M+2)^2 four-byte loads per window by 3 (M+2).
template <int M, int WT, int WK, int ALPHA, bool VEC>
__global__ void __launch_bounds__(64 * (M + 2) * WT * WK, 1)
wino_fused_mfma_kernel(const float* __restrict__ x, const float* __restrict__ U2, float* __restrict__ y, WinoGeom g)
{
    constexpr int n = M + 2, NP = n * n;
    constexpr int TB = 32 * WT, Z = 32 * WK, NBLK = WT * WK;
    constexpr int NWAVES = n * NBLK;
    constexpr int NCP = ALPHA / 2;                 // channel pairs per stage
    constexpr int UFLOATS = NCP * NP * Z * 2, VFLOATS = NCP * NP * TB * 2, STAGE = UFLOATS + VFLOATS;
    static_assert(ALPHA % 4 == 0 && ALPHA <= NWAVES && TB <= 64, "unsupported block");

    extern __shared__ float lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int row = wave % n, blk = wave / n, wt = blk % WT, wk = blk / WT;

    // blocks that share their sub-domains (the channel blocks of one strip) are neighbours on one XCD
    int bid = blockIdx.x;
    const int nblk = gridDim.x;
    if ((nblk & 7) == 0) bid = (bid & 7) * (nblk >> 3) + (bid >> 3);
    const int nbk = g.Kp / Z;
    const int kb = bid % nbk, tbk = bid / nbk;
    const int k0 = kb * Z, t0 = tbk * TB;

    // ---- this lane's transform task: sub-domain t0 + lane, channel `wave` of every stage ---------------------
    // The windows are read with buffer loads: an element outside the image (zero padding, a sub-domain past the
    // last one, a channel past C) gets a byte offset at or beyond the descriptor's size, for which the hardware
    // returns zero -- no masking arithmetic.  A lane's offset is a row part plus a column part; either may carry
    // the out-of-range mark, and two marks still add up to less than 2^32 (valid offsets stay below 2^30: checked
    // by the launcher).
    const bool task = wave < ALPHA && lane < TB;
    const int tpi = g.th * g.tw;                                   // sub-domains per image
    const int img0 = t0 / tpi;
    const int HW = g.H * g.W;
    typedef float vecm __attribute__((ext_vector_type(M)));
    typedef unsigned uvecm __attribute__((ext_vector_type(M)));
    constexpr unsigned OUTSIDE = 0x40000000u;
    constexpr int NCOL = VEC ? 3 : n;                              // VEC: left border, the M own columns, right border
    unsigned vrow[n], vcol[NCOL];                                  // byte offsets from channel 0 of the block's first image
    {
        int t = t0 + lane;
        const bool tv = task && t < g.tiles;
        if (!tv) t = t0;
        const int img = t / tpi, rem = t - img * tpi, ti = rem / g.tw, tj = rem - ti * g.tw;
        const int h0 = ti * M - g.pad, w0 = tj * M - g.pad;
#pragma unroll
        for (int i = 0; i < n; ++i) {
            const int h = h0 + i;
            vrow[i] = (tv && h >= 0 && h < g.H) ? 4u * (unsigned)((img - img0) * g.C * HW + h * g.W) : OUTSIDE;
        }
        if constexpr (VEC) {
            // pad = 1 and W a multiple of M: the own columns tj M .. tj M + M - 1 always lie inside the image
            vcol[0] = tj > 0 ? 4u * (unsigned)(tj * M - 1) : OUTSIDE;
            vcol[1] = 4u * (unsigned)(tj * M);
            vcol[2] = tj + 1 < g.tw ? 4u * (unsigned)(tj * M + M) : OUTSIDE;
        } else {
#pragma unroll
            for (int j = 0; j < n; ++j) {
                const int ww = w0 + j;
                vcol[j] = (ww >= 0 && ww < g.W) ? 4u * (unsigned)ww : OUTSIDE;
            }
        }
    }
    const float* xblk = x + (size_t)img0 * g.C * HW;

    float win[VEC ? 1 : n][VEC ? 1 : n];
    vecm mid[VEC ? n : 1];
    float wl[VEC ? n : 1], wr[VEC ? n : 1];
    auto load_windows = [&](int c0) {
        if (!task) return;
        const int c = c0 + wave;
        // the channel goes into the descriptor's base; a channel at or beyond C (the last stage of a C that is not a
        // multiple of ALPHA) gets a descriptor of size zero: every load returns zero
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(xblk + (size_t)(c < g.C ? c : 0) * HW), 0, c < g.C ? (int)OUTSIDE : 0, 0x00020000);
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < n; ++i) {
                wl[i] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, vrow[i] + vcol[0], 0, 0));
                if constexpr (M == 2) {
                    const uvecm q = __builtin_amdgcn_raw_buffer_load_b64(rs, vrow[i] + vcol[1], 0, 0);
                    mid[i][0] = __uint_as_float(q[0]);
                    mid[i][1] = __uint_as_float(q[1]);
                } else {
                    const uvecm q = __builtin_amdgcn_raw_buffer_load_b128(rs, vrow[i] + vcol[1], 0, 0);
#pragma unroll
                    for (int e = 0; e < M; ++e) mid[i][e] = __uint_as_float(q[e]);
                }
                wr[i] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, vrow[i] + vcol[2], 0, 0));
            }
        } else {
            // (the column parts pass through an empty asm statement so that the n * n sums are made here, stage by
            // stage, and not kept in n * n registers across the channel loop, where they would spill)
            unsigned col[n];
#pragma unroll
            for (int j = 0; j < n; ++j) {
                col[j] = vcol[j];
                asm volatile("" : "+v"(col[j]));
            }
#pragma unroll
            for (int i = 0; i < n; ++i)
#pragma unroll
                for (int j = 0; j < n; ++j)
                    win[i][j] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, vrow[i] + col[j], 0, 0));
        }
    };
    // B d column by column, then (B d) B^T row by row, each row stored as soon as it is complete.  Plain VALU
    // instructions run on the same pipeline as the fp32 MFMAs of the SIMD's other waves and wait for them, so the
    // transform is kept to its additions: no masks, no exchanges between lanes.
    auto transform_windows = [&](float* vbuf) {
        if (!task) return;
        float tmp[n][n];
        static_for<n>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            float col[n], out[n];
#pragma unroll
            for (int i = 0; i < n; ++i) {
                if constexpr (VEC) col[i] = j == 0 ? wl[i] : (j == n - 1 ? wr[i] : mid[i][j == 0 || j == n - 1 ? 0 : j - 1]);
                else col[i] = win[i][j];
            }
            mat_vec<M, UseB, n, n>(col, out);
#pragma unroll
            for (int i = 0; i < n; ++i) tmp[i][j] = out[i];
        });
        float* vp = vbuf + ((size_t)(wave >> 1) * NP * TB + lane) * 2 + (wave & 1);
        static_for<n>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            float out[n];
            mat_vec<M, UseB, n, n>(tmp[i], out);
#pragma unroll
            for (int j = 0; j < n; ++j) vp[(i * n + j) * TB * 2] = out[j];
        });
    };
    // the stage's slab of U2: NCP * NP rows of 2 Z floats, pitch 2 Kp
    const float* Ublk = U2 + (size_t)k0 * 2;
    // Every wave issues one load instruction: with nothing of its own in flight its LDS-base write does not wait.
    // The rest of the slab is left to the waves without a transform task: each further LDS-base write waits for the
    // load before it, and they wait while the others transform.
    auto issue_kernels = [&](int c0, float* ubuf) {
        constexpr int ROWS = NCP * NP, RPI = (Z / 2 <= 64 && 64 % (Z / 2) == 0) ? 64 / (Z / 2) : 1;
        constexpr int FIRST = (NWAVES * RPI < ROWS && ALPHA < NWAVES) ? NWAVES * RPI : ROWS;
        const float* src = Ublk + (size_t)(c0 >> 1) * NP * g.Kp * 2;
        stage_rows(src, g.Kp * 2, Z / 2, FIRST, ubuf, wave, NWAVES, lane);
        if constexpr (FIRST < ROWS) {
            if (wave >= ALPHA)
                stage_rows(src + (size_t)FIRST * g.Kp * 2, g.Kp * 2, Z / 2, ROWS - FIRST, ubuf + FIRST * Z * 2, wave - ALPHA,
                           NWAVES - ALPHA, lane);
        }
    };

    floatx16 acc[n];
#pragma unroll
    for (int p = 0; p < n; ++p)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[p][i] = 0.f;

    // operands of plane (row, p): lane half h reads channel pair 2 j + h
    const int aoff = (half * NP + row * n) * Z * 2 + (wk * 32 + l32) * 2;
    const int boff = UFLOATS + (half * NP + row * n) * TB * 2 + (wt * 32 + l32) * 2;

    const int nstages = (g.C + ALPHA - 1) / ALPHA;
    load_windows(0);
    issue_kernels(0, lds);
    lds_dma_wait_all();
    transform_windows(lds + UFLOATS);
    if (nstages > 1) load_windows(ALPHA);
    for (int s = 0; s < nstages; ++s) {
        lds_dma_wait_all();                 // this wave's part of U(s) has landed; so have the windows of stage s + 1
        __syncthreads();                    // V(s), U(s) complete; every wave is done with the other buffer
        const float* cur = lds + (s & 1) * STAGE;
        float* nxt = lds + ((s + 1) & 1) * STAGE;
        if (s + 1 < nstages) {
            issue_kernels((s + 1) * ALPHA, nxt);
            transform_windows(nxt + UFLOATS);
        }
        if (s + 2 < nstages) load_windows((s + 2) * ALPHA);
        // the n planes of this wave's row, per group of four channels: operands of the next group are fetched
        // while this one multiplies (two register sets)
        const float* ap = cur + aoff;
        const float* bp = cur + boff;
        constexpr int NGRP = ALPHA / 4;
        floatx2 fa[2][n], fb[2][n];
        auto fetch = [&](int set, int j) {
#pragma unroll
            for (int p = 0; p < n; ++p) {
                fa[set][p] = *reinterpret_cast<const floatx2*>(ap + ((2 * j) * NP + p) * Z * 2);
                fb[set][p] = *reinterpret_cast<const floatx2*>(bp + ((2 * j) * NP + p) * TB * 2);
            }
        };
        fetch(0, 0);
#pragma unroll
        for (int j = 0; j < NGRP; ++j) {
            if (j + 1 < NGRP) fetch((j + 1) & 1, j + 1);
#pragma unroll
            for (int p = 0; p < n; ++p)
                acc[p] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[j & 1][p][0], fb[j & 1][p][0], acc[p], 0, 0, 0);
#pragma unroll
            for (int p = 0; p < n; ++p)
                acc[p] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[j & 1][p][1], fb[j & 1][p][1], acc[p], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }

    // ---- output transform and store -------------------------------------------------------------------------
    // register r of an accumulator: channel 8 (r / 4) + 4 half + r % 4 of sub-domain l32 of the wave's block
    const int t = t0 + wt * 32 + l32;
    const bool tvalid = t < g.tiles;
    const int tt = tvalid ? t : t0;
    const int img = tt / tpi, rem = tt - img * tpi, ti = rem / g.tw, tj = rem - ti * g.tw;
    const size_t PQ = (size_t)g.P * g.Q;
    float* yt = y + (size_t)img * g.K * PQ + (size_t)(ti * M) * g.Q + tj * M;
    const int kbase = k0 + wk * 32 + 4 * half;
    const bool vec = (g.Q % M) == 0 && (reinterpret_cast<uintptr_t>(y) & (4 * M - 1)) == 0;
    auto store_tile = [&](int k, const float (&o)[M][M]) {
        if (!tvalid || k >= g.K) return;
        float* yk = yt + (size_t)k * PQ;
#pragma unroll
        for (int a = 0; a < M; ++a) {
            if (ti * M + a >= g.P) continue;
            if (vec) {
                vecm q;
#pragma unroll
                for (int b = 0; b < M; ++b) q[b] = o[a][b];
                *reinterpret_cast<vecm*>(yk + (size_t)a * g.Q) = q;
            } else {
#pragma unroll
                for (int b = 0; b < M; ++b)
                    if (tj * M + b < g.Q) yk[(size_t)a * g.Q + b] = o[a][b];
            }
        }
    };
    // The exchange runs in ROUNDS rounds of 16 / ROUNDS registers so that it fits the LDS.
    constexpr int ROUNDS = (NBLK * n * 16 * M * 64 * 4 > 160 * 1024) ? 2 : 1, RPR = 16 / ROUNDS;
    float* xch = lds + (size_t)blk * n * RPR * M * 64;               // [block][row][register of the round][b][lane]
    static_for<ROUNDS>([&](auto rc) {
        constexpr int r0 = decltype(rc)::value * RPR;
        __syncthreads();                                            // the staging buffers / the previous round are free
        static_for<RPR>([&](auto jc) {
            constexpr int r = r0 + decltype(jc)::value;
            float pi[n], tr[M];
#pragma unroll
            for (int c = 0; c < n; ++c) pi[c] = acc[c][r];
            mat_vec<M, UseA, M, n>(pi, tr);
            float* dst = xch + ((size_t)row * RPR + decltype(jc)::value) * M * 64 + lane;
#pragma unroll
            for (int b = 0; b < M; ++b) dst[b * 64] = tr[b];
        });
        __syncthreads();
        for (int jr = row; jr < RPR; jr += n) {
            float tin[n][M], o[M][M];
#pragma unroll
            for (int i = 0; i < n; ++i)
#pragma unroll
                for (int b = 0; b < M; ++b) tin[i][b] = xch[((size_t)i * RPR + jr) * M * 64 + b * 64 + lane];
            left_mul<M, UseA, M, n, M>(tin, o);
            const int r = r0 + jr;
            store_tile(kbase + 8 * (r >> 2) + (r & 3), o);
        }
    });
}

template <int M, int WT, int WK, int ALPHA, bool VEC>
hipError_t launch_fused_vec(const float* x, const float* U2, float* y, const WinoGeom& g, hipStream_t st)
{
    constexpr int n = M + 2, TB = 32 * WT, Z = 32 * WK, T = 64 * n * WT * WK;
    constexpr size_t stage = sizeof(float) * (size_t)(ALPHA / 2) * n * n * (Z + TB) * 2;
    constexpr size_t xch_all = sizeof(float) * (size_t)WT * WK * n * 16 * M * 64;
    constexpr size_t xch = xch_all > 160 * 1024 ? xch_all / 2 : xch_all;
    constexpr size_t shm = 2 * stage > xch ? 2 * stage : xch;
    static_assert(shm <= 160 * 1024, "block does not fit the LDS");
    if (g.tb != TB || g.z != Z || g.alpha != ALPHA || g.Kp % Z || g.Cp % ALPHA || g.Cp < g.C) return hipErrorInvalidValue;
    // per-lane byte offsets count from the first image of the block and stay below the out-of-range mark of the
    // window loads (2^30): a block spans at most TB / (sub-domains per image) + 2 images
    const long long tpi = (long long)g.th * g.tw;
    const long long span = ((TB + tpi - 1) / tpi + 2) * (long long)g.C * g.H * g.W * 4;
    if (span >= (1LL << 30)) return hipErrorInvalidValue;
    auto kern = wino_fused_mfma_kernel<M, WT, WK, ALPHA, VEC>;
    if (shm > 64 * 1024) {
        const hipError_t e = allow_large_lds((const void*)kern);
        if (e != hipSuccess) return e;
    }
    const long long grid_ll = (long long)(g.Kp / Z) * ((g.tiles + TB - 1) / TB);
    if (grid_ll > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid_ll), dim3(T), shm, st, x, U2, y, g);
    return hipGetLastError();
}

template <int M, int WT, int WK, int ALPHA>
hipError_t launch_fused_one(const float* x, const float* U2, float* y, const WinoGeom& g, hipStream_t st)
{
    const bool vec = g.pad == 1 && g.W % M == 0 && (reinterpret_cast<uintptr_t>(x) & (4 * M - 1)) == 0;
    return vec ? launch_fused_vec<M, WT, WK, ALPHA, true>(x, U2, y, g, st)
               : launch_fused_vec<M, WT, WK, ALPHA, false>(x, U2, y, g, st);
}

}  // namespace

hipError_t launch_wino_kernel_transform_paired(const float* w, float* U2, const WinoGeom& g, hipStream_t st)
{
    if (g.CpU & 1) return hipErrorInvalidValue;
    const size_t cnt = (size_t)g.CpU * g.Kp;
    const int grid = (int)((cnt + 255) / 256);
    switch (g.m) {
    case 2: hipLaunchKernelGGL(kernel_transform_paired<2>, dim3(grid), dim3(256), 0, st, w, U2, g.C, g.CpU, g.K, g.Kp); break;
    case 4: hipLaunchKernelGGL(kernel_transform_paired<4>, dim3(grid), dim3(256), 0, st, w, U2, g.C, g.CpU, g.K, g.Kp); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_wino_pair_relayout(const float* U, int rows, int cols, float* U2, const WinoGeom& g, hipStream_t st)
{
    const int planes = (g.m + 2) * (g.m + 2);
    const size_t cnt = (size_t)planes * g.Cp * g.Kp;
    if ((g.Cp & 1) || cnt >= ((size_t)1 << 31)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(pair_relayout_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, st, U, rows, cols, U2, g.Cp,
                       g.Kp, planes);
    return hipGetLastError();
}

// U2: the transformed kernels in the layout of launch_wino_kernel_transform_paired, g.Cp / 2 channel pairs of g.Kp
// columns.  g.m, g.tb, g.z and g.alpha select the block: F(2x2) runs the kernel of this file, F(4x4) the one of
// wino_fused_rows.hip.
hipError_t launch_wino_fused_mfma(const float* x, const float* U2, float* y, const WinoGeom& g, hipStream_t st)
{
    if (g.tiles < 1 || (reinterpret_cast<uintptr_t>(U2) & 15)) return hipErrorInvalidValue;
    if (g.m == 2 && g.tb == 64 && g.z == 64 && g.alpha == 8) return launch_fused_one<2, 2, 2, 8>(x, U2, y, g, st);
    if (g.m == 4) return launch_wino_fused_rows(x, U2, y, g, st);
    return hipErrorInvalidValue;
}

}  // namespace iolb
