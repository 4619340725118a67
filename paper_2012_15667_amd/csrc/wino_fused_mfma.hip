// Winograd F(m x m, 3 x 3), m in {2, 4}, for layers with many channels: the fused dataflow of Sec. 5.3 on the
// fp32 matrix cores.  One workgroup owns a block of tb sub-domains by z output channels and keeps ALL
// (m+2)^2 planes of its channel-summation temporaries (the Pi of step 3, Sec. 4.3) in accumulator registers
// for the whole channel loop; the transformed inputs (step 1) are made inside the workgroup, per stage of
// ALPHA channels, straight into the LDS buffer the products read, and the output transform (step 4) is
// applied to the accumulators in registers.  Neither the transformed inputs nor the temporaries ever reach
// memory: the layer reads x and the transformed kernels and writes y.
//
// Wave layout.  A 32 x 32 block (32 sub-domains by 32 channels) of one plane is one v_mfma_f32_32x32x2_f32
// accumulator of 16 registers.  The (m+2) rows of planes are dealt to RG "row groups"; a wave owns the
// (m+2)^2 / RG planes of its row group for one 32 x 32 block, so that, for a given (sub-domain, channel),
// every plane of the group sits in the same lane and register index of the wave's accumulators, and the
// output transform  Y = A Pi A^T = sum over rows i of  A[:, i] (Pi[i, :] A^T)  needs no data from other
// lanes.  With RG = 1 a wave finishes its outputs alone; with RG = 2 the two waves of a block each hold the
// partial sum over their rows, exchange half of it through LDS and add.
//
// Per stage the workgroup
//   - loads the (m+2) x (m+2) input windows of its sub-domains for the stage's channels from global memory
//     into registers (issued one stage ahead), transforms them (B d B^T) and writes them to LDS as
//     V[channel pair][plane][sub-domain][2];
//   - copies the stage's slab of the transformed kernels, U2[channel pair][plane][k][2], to LDS with
//     LDS-direct loads (issued one stage ahead);
//   - multiplies: per plane and group of four channels one 8-byte LDS read per operand feeds two MFMAs
//     (lane halves take channel pairs 2j and 2j + 1, so both halves use the same offsets).
// Two LDS buffers alternate; one barrier per stage.
#include <mutex>

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

// Partial output transform over the rows [R0, R0 + NR) of the planes: yp[a][b] = sum_{i in rows} A[a][i] *
// (sum_j pi[i - R0][j] * A[b][j]), coefficients folded at compile time.
template <int M, int R0, int NR>
__device__ __forceinline__ void output_rows(const float (&pi)[NR][M + 2], float (&yp)[M][M])
{
    constexpr int n = M + 2;
    float t[NR][M];
    right_mul_t<M, UseA, NR, n, M>(pi, t);
    static_for<M>([&](auto a) {
        static_for<M>([&](auto b) {
            float s = 0.f;
            bool first = true;
            static_for<NR>([&](auto i) {
                accumulate<M, UseA, decltype(a)::value, R0 + decltype(i)::value>(s, first, t[decltype(i)::value][decltype(b)::value]);
            });
            yp[decltype(a)::value][decltype(b)::value] = s;
        });
    });
}

// M: output tile edge.  RG: row groups (waves per 32 x 32 block).  WT x WK: blocks of the workgroup along
// sub-domains and channels (tb = 32 WT, z = 32 WK).  ALPHA: channels per stage.  CPT: channels per
// transform task (2: a lane transforms a channel pair and writes 8-byte pairs; 1: one channel, 4-byte writes).
// VEC (pad = 1, W a multiple of M, x aligned to 4 M bytes): a lane loads the M columns under its own
// sub-domain as one aligned vector per window row and takes the two border columns from its neighbour lanes
// (the sub-domains left and right of it; a border column outside the image is zero anyway), which replaces
// (M+2)^2 four-byte loads per window by M+2 wide ones; the first and the last lane of a block, whose
// neighbours belong to other workgroups, load their outer border column themselves.
template <int M, int RG, int WT, int WK, int ALPHA, int CPT, bool VEC>
__global__ void __launch_bounds__(64 * RG * WT * WK, 1)
wino_fused_mfma_kernel(const float* __restrict__ x, const float* __restrict__ U2, float* __restrict__ y, WinoGeom g)
{
    constexpr int n = M + 2, NP = n * n;
    constexpr int RPG = n / RG;                    // plane rows per wave
    constexpr int NPW = RPG * n;                   // planes per wave
    constexpr int TB = 32 * WT, Z = 32 * WK;
    constexpr int NWAVES = RG * WT * WK;
    constexpr int NCP = ALPHA / 2;                 // channel pairs per stage
    constexpr int NCG = ALPHA / CPT;               // transform task groups per stage (one wave each)
    constexpr int UFLOATS = NCP * NP * Z * 2, VFLOATS = NCP * NP * TB * 2, STAGE = UFLOATS + VFLOATS;
    static_assert(n % RG == 0 && ALPHA % 4 == 0 && NCG <= NWAVES && TB <= 64, "unsupported block");

    extern __shared__ float lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave % RG, blk = wave / RG, wt = blk % WT, wk = blk / WT;

    // blocks that share their sub-domains (the channel blocks of one strip) are neighbours on one XCD
    int bid = blockIdx.x;
    const int nblk = gridDim.x;
    if ((nblk & 7) == 0) bid = (bid & 7) * (nblk >> 3) + (bid >> 3);
    const int nbk = g.Kp / Z;
    const int kb = bid % nbk, tbk = bid / nbk;
    const int k0 = kb * Z, t0 = tbk * TB;

    // ---- this lane's transform task: sub-domain t0 + lane, channel group `wave` of every stage -------------
    const bool task = wave < NCG && lane < TB;
    const int tpi = g.th * g.tw;                                   // sub-domains per image
    const int img0 = t0 / tpi;
    const int HW = g.H * g.W;
    typedef float vecm __attribute__((ext_vector_type(M)));
    unsigned voff[VEC ? 1 : n][VEC ? 1 : n];                       // scalar path: byte offsets of the window elements
    unsigned vrow[VEC ? n : 1];                                    // vector path: byte offsets of the own columns per row
    bool rv[n], cv[n];
    bool edge_lane = false;
    int edge_delta = 0;
    {
        int t = t0 + lane;
        const bool tv = task && t < g.tiles;
        if (!tv) t = t0;
        const int img = t / tpi, rem = t - img * tpi, ti = rem / g.tw, tj = rem - ti * g.tw;
        const int h0 = ti * M - g.pad, w0 = tj * M - g.pad;
        unsigned ro[n], co[n];
#pragma unroll
        for (int i = 0; i < n; ++i) {
            const int h = h0 + i, ww = w0 + i;
            rv[i] = tv && h >= 0 && h < g.H;
            cv[i] = ww >= 0 && ww < g.W;
            ro[i] = (unsigned)((img - img0) * g.C * HW + (h < 0 ? 0 : (h >= g.H ? g.H - 1 : h)) * g.W);
            co[i] = (unsigned)(ww < 0 ? 0 : (ww >= g.W ? g.W - 1 : ww));
        }
        if constexpr (VEC) {
#pragma unroll
            for (int i = 0; i < n; ++i) vrow[i] = 4u * (ro[i] + (unsigned)(tj * M));
            // the block's first lane has no left neighbour in the wave, its last lane no right one
            const bool first = lane == 0 && tj > 0, last = lane == TB - 1 && tj + 1 < g.tw;
            edge_lane = tv && (first || last);
            edge_delta = first ? -4 : 4 * M;
        } else {
#pragma unroll
            for (int i = 0; i < n; ++i)
#pragma unroll
                for (int j = 0; j < n; ++j) voff[i][j] = 4u * (ro[i] + co[j]);
        }
    }
    const float* xblk = x + (size_t)img0 * g.C * HW;

    float win[VEC ? 1 : CPT][VEC ? 1 : n][VEC ? 1 : n];
    vecm mid[VEC ? CPT : 1][VEC ? n : 1];
    float edge[VEC ? CPT : 1][VEC ? n : 1];
    // channels at or beyond C (the last stage of a C that is not a multiple of ALPHA) read channel C - 1 and
    // are zeroed in the transform
    auto load_windows = [&](int c0) {
        if (!task) return;
#pragma unroll
        for (int e = 0; e < CPT; ++e) {
            const int c = c0 + wave * CPT + e;
            const char* xc = reinterpret_cast<const char*>(xblk + (size_t)(c < g.C ? c : g.C - 1) * HW);
            if constexpr (VEC) {
#pragma unroll
                for (int i = 0; i < n; ++i) mid[e][i] = *reinterpret_cast<const vecm*>(xc + vrow[i]);
            } else {
#pragma unroll
                for (int i = 0; i < n; ++i)
#pragma unroll
                    for (int j = 0; j < n; ++j) win[e][i][j] = *reinterpret_cast<const float*>(xc + voff[i][j]);
            }
        }
        if constexpr (VEC) {
            if (edge_lane) {
#pragma unroll
                for (int e = 0; e < CPT; ++e) {
                    const int c = c0 + wave * CPT + e;
                    const char* xc = reinterpret_cast<const char*>(xblk + (size_t)(c < g.C ? c : g.C - 1) * HW);
#pragma unroll
                    for (int i = 0; i < n; ++i) edge[e][i] = *reinterpret_cast<const float*>(xc + vrow[i] + edge_delta);
                }
            }
        }
    };
    auto transform_windows = [&](int c0, float* vbuf) {
        if (!task) return;
        if constexpr (CPT == 1) {
            // One channel per lane, written for few live registers (the accumulators leave little room when
            // many waves share a SIMD): first B d column by column, then (B d) B^T row by row, each row stored
            // as soon as it is complete.
            const bool cvalid = c0 + wave < g.C;
            float tmp[n][n];
            static_for<n>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                float col[n], out[n];
#pragma unroll
                for (int i = 0; i < n; ++i) {
                    float vin;
                    if constexpr (VEC) {
                        if constexpr (j == 0) {
                            const float own_last = mid[0][i][M - 1];
                            vin = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (lane - 1), __float_as_int(own_last)));
                            if (lane == 0) vin = edge[0][i];
                        } else if constexpr (j == n - 1) {
                            const float own_first = mid[0][i][0];
                            vin = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (lane + 1), __float_as_int(own_first)));
                            if (lane == TB - 1) vin = edge[0][i];
                        } else {
                            vin = mid[0][i][j - 1];
                        }
                    } else {
                        vin = win[0][i][j];
                    }
                    col[i] = (cvalid && rv[i] && cv[j]) ? vin : 0.f;
                }
                mat_vec<M, UseB, n, n>(col, out);
#pragma unroll
                for (int i = 0; i < n; ++i) tmp[i][j] = out[i];
                __builtin_amdgcn_sched_barrier(0);
            });
            float* vp = vbuf + ((size_t)(wave >> 1) * NP * TB + lane) * 2 + (wave & 1);
            static_for<n>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                float out[n];
                mat_vec<M, UseB, n, n>(tmp[i], out);
#pragma unroll
                for (int j = 0; j < n; ++j) vp[(i * n + j) * TB * 2] = out[j];
                __builtin_amdgcn_sched_barrier(0);
            });
            return;
        }
        float v[CPT][n][n];
#pragma unroll
        for (int e = 0; e < CPT; ++e) {
            const bool cvalid = c0 + wave * CPT + e < g.C;
            float d[n][n], tmp[n][n];
            if constexpr (VEC) {
#pragma unroll
                for (int i = 0; i < n; ++i) {
                    // the value of the lane below / above (ds_bpermute: a lane reads the lane whose byte index it
                    // gives).  The components are copied to scalars first: a bit cast applied directly to a vector
                    // element reads element 0.
                    const float own_last = mid[e][i][M - 1], own_first = mid[e][i][0];
                    float left = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (lane - 1), __float_as_int(own_last)));
                    float right = __int_as_float(__builtin_amdgcn_ds_bpermute(4 * (lane + 1), __float_as_int(own_first)));
                    if (lane == 0) left = edge[e][i];
                    if (lane == TB - 1) right = edge[e][i];
                    const bool row = cvalid && rv[i];
                    d[i][0] = (row && cv[0]) ? left : 0.f;
#pragma unroll
                    for (int j = 0; j < M; ++j) d[i][j + 1] = row ? mid[e][i][j] : 0.f;
                    d[i][n - 1] = (row && cv[n - 1]) ? right : 0.f;
                }
            } else {
#pragma unroll
                for (int i = 0; i < n; ++i)
#pragma unroll
                    for (int j = 0; j < n; ++j) d[i][j] = (cvalid && rv[i] && cv[j]) ? win[e][i][j] : 0.f;
            }
            left_mul<M, UseB, n, n, n>(d, tmp);
            right_mul_t<M, UseB, n, n, n>(tmp, v[e]);
        }
        if constexpr (CPT == 2) {
            float* vp = vbuf + ((size_t)wave * NP * TB + lane) * 2;
#pragma unroll
            for (int i = 0; i < n; ++i)
#pragma unroll
                for (int j = 0; j < n; ++j)
                    *reinterpret_cast<floatx2*>(vp + (i * n + j) * TB * 2) = floatx2{v[0][i][j], v[1][i][j]};
        } else {
            float* vp = vbuf + ((size_t)(wave >> 1) * NP * TB + lane) * 2 + (wave & 1);
#pragma unroll
            for (int i = 0; i < n; ++i)
#pragma unroll
                for (int j = 0; j < n; ++j) vp[(i * n + j) * TB * 2] = v[0][i][j];
        }
    };
    // the stage's slab of U2: NCP * NP rows of 2 Z floats, pitch 2 Kp
    const float* Ublk = U2 + (size_t)k0 * 2;
    auto issue_kernels = [&](int c0, float* ubuf) {
        stage_rows(Ublk + (size_t)(c0 >> 1) * NP * g.Kp * 2, g.Kp * 2, Z / 2, NCP * NP, ubuf, wave, NWAVES, lane);
    };

    floatx16 acc[NPW];
#pragma unroll
    for (int p = 0; p < NPW; ++p)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[p][i] = 0.f;

    // operands of plane p (row grp * RPG + p / n): lane half h reads channel pair 2 j + h
    const int plane0 = grp * NPW;
    const int aoff = (half * NP + plane0) * Z * 2 + (wk * 32 + l32) * 2;
    const int boff = UFLOATS + (half * NP + plane0) * TB * 2 + (wt * 32 + l32) * 2;

    const int nstages = (g.C + ALPHA - 1) / ALPHA;
    load_windows(0);
    issue_kernels(0, lds);
    lds_dma_wait_all();
    transform_windows(0, lds + UFLOATS);
    if (nstages > 1) load_windows(ALPHA);
    for (int s = 0; s < nstages; ++s) {
        lds_dma_wait_all();                 // this wave's part of U(s) has landed; so have the windows of stage s + 1
        __syncthreads();                    // V(s), U(s) complete; every wave is done with the other buffer
        const float* cur = lds + (s & 1) * STAGE;
        float* nxt = lds + ((s + 1) & 1) * STAGE;
        if (s + 1 < nstages) {
#ifndef EXP_NO_U
            issue_kernels((s + 1) * ALPHA, nxt);
#endif
#ifndef EXP_NO_TRANSFORM
            transform_windows((s + 1) * ALPHA, nxt + UFLOATS);
#endif
        }
#ifndef EXP_NO_WINLOAD
        if (s + 2 < nstages) load_windows((s + 2) * ALPHA);
#endif
#ifndef EXP_NO_MFMA
        // Operands of a group of GP planes are fetched while the previous group multiplies (two register sets).
        const float* ap = cur + aoff;
        const float* bp = cur + boff;
        constexpr int GP = NPW % 4 == 0 ? 4 : 3, NGRP = (ALPHA / 4) * (NPW / GP);
        static_assert(NPW % GP == 0, "planes per wave must split into operand groups");
        floatx2 fa[2][GP], fb[2][GP];
        auto fetch = [&](int set, int grpi) {
            const int j = grpi / (NPW / GP), p0 = (grpi % (NPW / GP)) * GP;
#pragma unroll
            for (int q = 0; q < GP; ++q) {
                fa[set][q] = *reinterpret_cast<const floatx2*>(ap + ((2 * j) * NP + p0 + q) * Z * 2);
                fb[set][q] = *reinterpret_cast<const floatx2*>(bp + ((2 * j) * NP + p0 + q) * TB * 2);
            }
        };
        fetch(0, 0);
#pragma unroll
        for (int gi = 0; gi < NGRP; ++gi) {
            if (gi + 1 < NGRP) fetch((gi + 1) & 1, gi + 1);
            const int p0 = (gi % (NPW / GP)) * GP;
#pragma unroll
            for (int q = 0; q < GP; ++q)
                acc[p0 + q] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[gi & 1][q][0], fb[gi & 1][q][0], acc[p0 + q], 0, 0, 0);
#pragma unroll
            for (int q = 0; q < GP; ++q)
                acc[p0 + q] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[gi & 1][q][1], fb[gi & 1][q][1], acc[p0 + q], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
#endif
    }

    // ---- output transform and store -------------------------------------------------------------------------
    // register i of an accumulator: channel 8 (i / 4) + 4 half + i % 4 of sub-domain l32 of the wave's block
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
                typedef float vecm __attribute__((ext_vector_type(M)));
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
    auto partial = [&](auto ic, float (&o)[M][M]) {
        constexpr int i = decltype(ic)::value;
        float pi[RPG][n];
#pragma unroll
        for (int r = 0; r < RPG; ++r)
#pragma unroll
            for (int c = 0; c < n; ++c) pi[r][c] = acc[r * n + c][i];
        if (grp == 0) output_rows<M, 0, RPG>(pi, o);
        else if constexpr (RG == 2) output_rows<M, RPG, RPG>(pi, o);
    };
    if constexpr (RG == 1) {
        static_for<16>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            float o[M][M];
            partial(ic, o);
            store_tile(kbase + 8 * (i >> 2) + (i & 3), o);
        });
    } else if constexpr (RG == 2) {
        // The two waves of a block each hold the sum over their plane rows.  Group 0 finishes registers 0..7,
        // group 1 registers 8..15: each writes the partial sums of the other's registers to LDS (the staging
        // buffers are free by now), then adds what the other wrote to its own.
        __syncthreads();                                            // every wave is done with the staging buffers
        float* xch = lds + (size_t)blk * 2 * 8 * M * M * 64;         // [group that reads][8][M*M][64]
        static_for<8>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            float o[M][M];
            if (grp == 0) partial(std::integral_constant<int, 8 + j>{}, o);
            else          partial(std::integral_constant<int, j>{}, o);
            float* dst = xch + ((size_t)(1 - grp) * 8 + j) * M * M * 64 + lane;
#pragma unroll
            for (int a = 0; a < M; ++a)
#pragma unroll
                for (int b = 0; b < M; ++b) dst[(a * M + b) * 64] = o[a][b];
        });
        __syncthreads();
        static_for<8>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            float o[M][M];
            if (grp == 0) partial(std::integral_constant<int, j>{}, o);
            else          partial(std::integral_constant<int, 8 + j>{}, o);
            const float* src = xch + ((size_t)grp * 8 + j) * M * M * 64 + lane;
#pragma unroll
            for (int a = 0; a < M; ++a)
#pragma unroll
                for (int b = 0; b < M; ++b) o[a][b] += src[(a * M + b) * 64];
            const int i = grp == 0 ? j : 8 + j;
            store_tile(kbase + 8 * (i >> 2) + (i & 3), o);
        });
    } else {
        // One wave per plane row (RG = m + 2).  The output transform is done in two halves around an exchange:
        // wave i applies A^T from the right to its row, T[i][b] = sum_j Pi[i][j] A[b][j], and writes the m values
        // per (register, lane) to LDS; then the 16 registers are dealt to the waves of the block, and the wave
        // that finishes register r reads the (m+2) x m values T[.][.] of its lanes, applies A from the left and
        // stores.  The exchange runs in ROUNDS rounds of 16 / ROUNDS registers so that it fits the LDS.
        static_assert(RG == n, "row groups: 1, 2 or one per plane row");
        constexpr int NBLK = WT * WK;
        constexpr int ROUNDS = (NBLK * n * 16 * M * 64 * 4 > 160 * 1024) ? 2 : 1, RPR = 16 / ROUNDS;
        float* xch = lds + (size_t)blk * n * RPR * M * 64;           // [block][row][register of the round][b][lane]
        static_for<ROUNDS>([&](auto rc) {
            constexpr int r0 = decltype(rc)::value * RPR;
            __syncthreads();                                        // the staging buffers / the previous round are free
            static_for<RPR>([&](auto jc) {
                constexpr int r = r0 + decltype(jc)::value;
                float pi[1][n], tr[1][M];
#pragma unroll
                for (int c = 0; c < n; ++c) pi[0][c] = acc[c][r];
                right_mul_t<M, UseA, 1, n, M>(pi, tr);
                float* dst = xch + ((size_t)grp * RPR + decltype(jc)::value) * M * 64 + lane;
#pragma unroll
                for (int b = 0; b < M; ++b) dst[b * 64] = tr[0][b];
            });
            __syncthreads();
            for (int jr = grp; jr < RPR; jr += n) {
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
}

template <int M, int RG, int WT, int WK, int ALPHA, int CPT, bool VEC>
hipError_t launch_fused_vec(const float* x, const float* U2, float* y, const WinoGeom& g, hipStream_t st)
{
    constexpr int n = M + 2, TB = 32 * WT, Z = 32 * WK, T = 64 * RG * WT * WK;
    constexpr size_t stage = sizeof(float) * (size_t)(ALPHA / 2) * n * n * (Z + TB) * 2;
    constexpr size_t xch_all = sizeof(float) * (size_t)WT * WK * n * 16 * M * 64;       // one wave per plane row
    constexpr size_t xch = RG == 1 ? 0 : RG == 2 ? sizeof(float) * (size_t)WT * WK * 2 * 8 * M * M * 64
                                                 : (xch_all > 160 * 1024 ? xch_all / 2 : xch_all);
    constexpr size_t shm = 2 * stage > xch ? 2 * stage : xch;
    static_assert(shm <= 160 * 1024, "block does not fit the LDS");
    if (g.tb != TB || g.z != Z || g.alpha != ALPHA || g.Kp % Z || g.Cp % ALPHA || g.Cp < g.C) return hipErrorInvalidValue;
    // per-lane byte offsets are 32 bits from the first image of the block: a block spans at most
    // TB / (sub-domains per image) + 2 images
    const long long tpi = (long long)g.th * g.tw;
    const long long span = ((TB + tpi - 1) / tpi + 2) * (long long)g.C * g.H * g.W * 4;
    if (span >= (1LL << 32)) return hipErrorInvalidValue;
    auto kern = wino_fused_mfma_kernel<M, RG, WT, WK, ALPHA, CPT, VEC>;
    static std::once_flag raised;
    static hipError_t raise_rc = hipSuccess;
    std::call_once(raised, [&] {
        if (shm > 64 * 1024)
            raise_rc = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    });
    if (raise_rc != hipSuccess) return raise_rc;
    const long long grid_ll = (long long)(g.Kp / Z) * ((g.tiles + TB - 1) / TB);
    if (grid_ll > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid_ll), dim3(T), shm, st, x, U2, y, g);
    return hipGetLastError();
}

template <int M, int RG, int WT, int WK, int ALPHA, int CPT>
hipError_t launch_fused_one(const float* x, const float* U2, float* y, const WinoGeom& g, hipStream_t st)
{
    const bool vec = g.pad == 1 && g.W % M == 0 && (reinterpret_cast<uintptr_t>(x) & (4 * M - 1)) == 0;
    return vec ? launch_fused_vec<M, RG, WT, WK, ALPHA, CPT, true>(x, U2, y, g, st)
               : launch_fused_vec<M, RG, WT, WK, ALPHA, CPT, false>(x, U2, y, g, st);
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

// U2: the transformed kernels in the layout of launch_wino_kernel_transform_paired, g.Cp / 2 channel pairs.
// g.waves_m = RG * WK and g.waves_n = WT select the instantiation together with g.tb, g.z and g.alpha.
hipError_t launch_wino_fused_mfma(const float* x, const float* U2, float* y, const WinoGeom& g, hipStream_t st)
{
    if (g.tiles < 1 || (reinterpret_cast<uintptr_t>(U2) & 15)) return hipErrorInvalidValue;
    if (g.m == 2 && g.tb == 64 && g.z == 64 && g.alpha == 8) {
        if (g.waves_m == 2) return launch_fused_one<2, 1, 2, 2, 8, 2>(x, U2, y, g, st);
        if (g.waves_m == 4) return launch_fused_one<2, 2, 2, 2, 8, 2>(x, U2, y, g, st);
        if (g.waves_m == 8) return launch_fused_one<2, 4, 2, 2, 8, 1>(x, U2, y, g, st);
    }
    if (g.m == 4 && g.tb == 32 && g.z == 64 && g.alpha == 4) {
        if (g.waves_m == 4) return launch_fused_one<4, 2, 1, 2, 4, 1>(x, U2, y, g, st);
        if (g.waves_m == 12) return launch_wino_fused_rows(x, U2, y, g, st);
    }
    if (g.m == 2 && g.tb == 64 && g.z == 64 && g.alpha == 4 && g.waves_m == 8) return launch_wino_fused_rows(x, U2, y, g, st);
    return hipErrorInvalidValue;
}

}  // namespace iolb
