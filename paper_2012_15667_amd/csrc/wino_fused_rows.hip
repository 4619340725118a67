// Winograd F(m x m, 3 x 3) fused on the matrix cores (dataflow of Sec. 5.3), "row waves" variant: the workgroup
// keeps all (m+2)^2 planes of its tb x z block of channel-summation temporaries in accumulator registers, ONE
// WAVE PER PLANE ROW and 32 x 32 block, so that a compute unit runs 12 to 16 light waves (3 or 4 per SIMD) that
// hide each other's LDS traffic, loads and barriers behind matrix-core work.  (Not the transform arithmetic:
// plain VALU instructions and fp32 MFMAs share one pipeline per SIMD, so every vector instruction is paid in
// matrix time -- hence buffer loads whose range check supplies the zero padding, and scalar stage bases.)
//
// Every thread takes an equal share of the input transform (step 1 of Sec. 4.3), which runs in two halves
// through an LDS scratch buffer so that no thread ever holds a whole window:
//   pass 1  a thread owns one window COLUMN (sub-domain, channel, j): it loads the m+2 pixels of the column
//           from global memory (one stage ahead), multiplies by B from the left and writes the m+2 results to
//           the scratch buffer;
//   pass 2  a thread owns one ROW (sub-domain, channel, i) of B d: it reads the m+2 values from the scratch
//           buffer, multiplies by B^T from the right and writes the row of transformed values into the
//           product's LDS stage, V[channel pair][plane][sub-domain][2].
// The transformed kernels U2[channel pair][plane][k][2] are copied to the stage through registers, loaded one
// stage ahead.  The product (steps 2, 3)
// reads 8-byte operand pairs (lane halves take channel pairs 2j and 2j + 1) and issues two MFMAs per read pair.
// The output transform (step 4) is split around an exchange: each wave applies A^T from the right to its plane
// row, T[i][b] = sum_j Pi[i][j] A[b][j]; the m values per (register, lane) go through LDS; the wave that
// finishes register r then applies A from the left over the m+2 rows and stores.
//
// Buffers: two product stages (U2 slab + V) and two scratch buffers alternate; one barrier per stage.
#include "kernels.h"
#include "wino_mats.h"
#include "wino_transform.h"

namespace iolb {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// out[ROWS] = Mx[ROWS][IN] * in[IN], Mx = Sel's matrix of Mats<M>, coefficients folded at compile time.
template <int M, class Sel, int ROWS, int IN>
__device__ __forceinline__ void rows_mat_vec(const float (&in)[IN], float (&out)[ROWS])
{
    static_for<ROWS>([&](auto i) {
        float s = 0.f;
        bool first = true;
        static_for<IN>([&](auto k) { accumulate<M, Sel, decltype(i)::value, decltype(k)::value>(s, first, in[k]); });
        out[decltype(i)::value] = s;
    });
}

// M: output tile edge.  WT x WK: 32 x 32 blocks of the workgroup along sub-domains and channels (tb = 32 WT,
// z = 32 WK).  ALPHA: channels per stage.
template <int M, int WT, int WK, int ALPHA>
__global__ void __launch_bounds__(64 * (M + 2) * WT * WK, 1)
wino_rows_kernel(const float* __restrict__ x, const float* __restrict__ U2, float* __restrict__ y, WinoGeom g)
{
    constexpr int n = M + 2, NP = n * n;
    constexpr int TB = 32 * WT, Z = 32 * WK, NBLK = WT * WK;
    constexpr int NWAVES = n * NBLK, T = 64 * NWAVES;
    constexpr int NCP = ALPHA / 2;
    constexpr int UFLOATS = NCP * NP * Z * 2, VFLOATS = NCP * NP * TB * 2, STAGE = UFLOATS + VFLOATS;
    constexpr int SP = NP + 1;                                  // scratch pitch per window: odd, so lanes that walk over
                                                                // sub-domains hit different banks
    constexpr int SCRATCH = ALPHA * TB * SP;
    constexpr int NTASK = ALPHA * TB * n, NT = NTASK / T;       // column (pass 1) and row (pass 2) tasks per stage / thread
    static_assert(NTASK % T == 0 && (n * TB) % 64 == 0 && ALPHA % 4 == 0, "unsupported block");

    extern __shared__ float lds[];
    float* const scratch0 = lds + 2 * STAGE;
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

    const int tpi = g.th * g.tw;                                // sub-domains per image
    const int img0 = t0 / tpi;
    const int HW = g.H * g.W;
    const float* xblk = x + (size_t)img0 * g.C * HW;

    // ---- pass 1 geometry: task q = tid + it * T  ->  (channel q / (n TB), sub-domain (q / n) % TB, column q % n) ----
    // The pixels are read with buffer loads: one outside the image (zero padding, a sub-domain past the last one, a
    // channel past C) gets a byte offset at or beyond the descriptor's size, for which the hardware returns zero --
    // no masking arithmetic (plain VALU instructions share the pipeline of the fp32 MFMAs: each one costs the SIMD
    // matrix time).  Valid offsets stay below the mark (checked by the launcher).
    constexpr unsigned OUTSIDE = 0x40000000u;
    unsigned coff[NT][n];              // byte offset of the column's pixel in window row i, from channel 0 of the block's first image
    int p1_dst[NT];                    // scratch offset of (window, column)
    int p1_ch[NT];                     // channel of the task within its stage (the same for all lanes of a wave)
#pragma unroll
    for (int it = 0; it < NT; ++it) {
        const int q = tid + it * T;
        const int j = q % n, tl = (q / n) % TB;
        int t = t0 + tl;
        const bool tv = t < g.tiles;
        if (!tv) t = t0;
        const int img = t / tpi, rem = t - img * tpi, ti = rem / g.tw, tj = rem - ti * g.tw;
        const int h0 = ti * M - g.pad, ww = tj * M - g.pad + j;
        const bool cvalid = tv && ww >= 0 && ww < g.W;
#pragma unroll
        for (int i = 0; i < n; ++i) {
            const int h = h0 + i;
            coff[it][i] = (cvalid && h >= 0 && h < g.H) ? 4u * (unsigned)((img - img0) * g.C * HW + h * g.W + ww) : OUTSIDE;
        }
        p1_dst[it] = ((q / (n * TB)) * TB + tl) * SP + j;
        p1_ch[it] = __builtin_amdgcn_readfirstlane(q / (n * TB));
    }
    // ---- pass 2 geometry: task q -> (channel q / (n TB), window row (q / TB) % n, sub-domain q % TB) --------------
    int p2_src[NT], p2_dst[NT];
#pragma unroll
    for (int it = 0; it < NT; ++it) {
        const int q = tid + it * T;
        const int tl = q % TB, i = (q / TB) % n, c = q / (n * TB);
        p2_src[it] = (c * TB + tl) * SP + i * n;
        p2_dst[it] = (((c >> 1) * NP + i * n) * TB + tl) * 2 + (c & 1);
    }

    float colv[NT][n];
    // the channel goes into the descriptor's base; a channel at or beyond C (the last stage of a C that is not a
    // multiple of ALPHA) gets a descriptor of size zero: every load returns zero
    auto load_columns = [&](int c0) {
#pragma unroll
        for (int it = 0; it < NT; ++it) {
            const int c = c0 + p1_ch[it];
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<float*>(xblk + (size_t)(c < g.C ? c : 0) * HW), 0, c < g.C ? (int)OUTSIDE : 0, 0x00020000);
#pragma unroll
            for (int i = 0; i < n; ++i) colv[it][i] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rs, coff[it][i], 0, 0));
        }
    };
    auto pass1 = [&](float* sbuf) {
#pragma unroll
        for (int it = 0; it < NT; ++it) {
            float out[n];
            rows_mat_vec<M, UseB, n, n>(colv[it], out);
            float* dst = sbuf + p1_dst[it];
#pragma unroll
            for (int i = 0; i < n; ++i) dst[i * n] = out[i];
        }
    };
    auto pass2 = [&](const float* sbuf, float* vbuf) {
#pragma unroll
        for (int it = 0; it < NT; ++it) {
            float rowv[n], out[n];
            const float* src = sbuf + p2_src[it];
#pragma unroll
            for (int j = 0; j < n; ++j) rowv[j] = src[j];
            rows_mat_vec<M, UseB, n, n>(rowv, out);
            float* dst = vbuf + p2_dst[it];
#pragma unroll
            for (int j = 0; j < n; ++j) dst[j * TB * 2] = out[j];
        }
    };
    // The stage's slab of U2 (NCP * NP rows of 2 Z floats, pitch 2 Kp) goes through registers: every thread
    // loads NU 16-byte pieces one stage ahead and writes them to the stage buffer when the stage is prepared.
    typedef float floatx4 __attribute__((ext_vector_type(4)));
    constexpr int NU = UFLOATS / 4 / T;
    static_assert(UFLOATS % (4 * T) == 0, "the kernel slab must split evenly over the threads");
    unsigned uoff[NU];
#pragma unroll
    for (int it = 0; it < NU; ++it) {
        const int e = tid + it * T;
        uoff[it] = 4u * (unsigned)((e / (Z / 2)) * g.Kp * 2 + (e % (Z / 2)) * 4);
    }
    const float* Ublk = U2 + (size_t)k0 * 2;
    floatx4 ureg[NU];
    // (buffer loads: the stage's base is a scalar and the lane's offset goes in as it is -- no 64-bit address
    // arithmetic on the vector unit)
    typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
    auto load_kernels = [&](int c0) {
        const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<float*>(Ublk + (size_t)(c0 >> 1) * NP * g.Kp * 2), 0, 0x7fffffff, 0x00020000);
#pragma unroll
        for (int it = 0; it < NU; ++it) {
            const uintx4 q = __builtin_amdgcn_raw_buffer_load_b128(rs, uoff[it], 0, 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) ureg[it][e] = __uint_as_float(q[e]);
        }
    };
    auto store_kernels = [&](float* ubuf) {
#pragma unroll
        for (int it = 0; it < NU; ++it) *reinterpret_cast<floatx4*>(ubuf + (size_t)(tid + it * T) * 4) = ureg[it];
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
    // Stage k is PREPARED (U(k) written from the registers it was loaded into an interval earlier, V(k) written
    // by pass 2, the scratch of stage k + 1 written by pass 1, U(k + 1) and the columns of stage k + 2 requested)
    // in the barrier interval before the one that MULTIPLIES it.  The waves of a SIMD (w, w + 4, w + 8, ...) take
    // the two halves of an interval in opposite orders -- "early" waves prepare first, "late" waves multiply
    // first -- so that the matrix core always has a wave that multiplies while another one transforms.
    const bool late = (wave >> 2) & 1;
    auto prepare = [&](int k) {
        if (k >= 1 && k < nstages) {
            float* buf = lds + (k & 1) * STAGE;
            store_kernels(buf);
            pass2(scratch0 + (k & 1) * SCRATCH, buf + UFLOATS);
        }
        if (k >= 1 && k + 1 < nstages) load_kernels((k + 1) * ALPHA);
        if (k >= 1 && k + 1 < nstages) pass1(scratch0 + ((k + 1) & 1) * SCRATCH);
        if (k >= 1 && k + 2 < nstages) load_columns((k + 2) * ALPHA);
    };
    // the n planes of this wave's row, per group of four channels: operands of the next group are fetched while
    // this one multiplies
    auto multiply = [&](const float* cur) {
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
    };

    // prologue: stage 0 prepared by everybody in the same order
    load_columns(0);
    load_kernels(0);
    pass1(scratch0);
    if (nstages > 1) load_columns(ALPHA);
    store_kernels(lds);
    if (nstages > 1) load_kernels(ALPHA);
    __syncthreads();
    pass2(scratch0, lds + UFLOATS);
    if (nstages > 1) pass1(scratch0 + SCRATCH);
    if (nstages > 2) load_columns(2 * ALPHA);
    for (int s = 0; s < nstages; ++s) {
        // the barrier that opens interval s: everything stage s needs is complete, stage s - 1 is consumed
        if (!late) __syncthreads();
        prepare(late ? s : s + 1);
        if (late) __syncthreads();
        multiply(lds + (s & 1) * STAGE);
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
            rows_mat_vec<M, UseA, M, n>(pi, tr);
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

template <int M, int WT, int WK, int ALPHA>
hipError_t launch_rows_one(const float* x, const float* U2, float* y, const WinoGeom& g, hipStream_t st)
{
    constexpr int n = M + 2, TB = 32 * WT, Z = 32 * WK, T = 64 * n * WT * WK;
    constexpr size_t stage = sizeof(float) * (size_t)(ALPHA / 2) * n * n * (Z + TB) * 2;
    constexpr size_t scratch = sizeof(float) * (size_t)ALPHA * TB * (n * n + 1);
    constexpr size_t xch_all = sizeof(float) * (size_t)WT * WK * n * 16 * M * 64;
    constexpr size_t xch = xch_all > 160 * 1024 ? xch_all / 2 : xch_all;
    constexpr size_t main_bytes = 2 * stage + 2 * scratch;
    constexpr size_t shm = main_bytes > xch ? main_bytes : xch;
    static_assert(shm <= 160 * 1024, "block does not fit the LDS");
    if (g.tb != TB || g.z != Z || g.alpha != ALPHA || g.Kp % Z || g.Cp % ALPHA || g.Cp < g.C) return hipErrorInvalidValue;
    // per-lane byte offsets count from the first image of the block and stay below the out-of-range mark of the
    // window loads (2^30): a block spans at most
    // TB / (sub-domains per image) + 2 images
    const long long tpi = (long long)g.th * g.tw;
    const long long span = ((TB + tpi - 1) / tpi + 2) * (long long)g.C * g.H * g.W * 4;
    if (span >= (1LL << 30)) return hipErrorInvalidValue;
    auto kern = wino_rows_kernel<M, WT, WK, ALPHA>;
    if (shm > 64 * 1024) {
        const hipError_t e = allow_large_lds((const void*)kern);
        if (e != hipSuccess) return e;
    }
    const long long grid_ll = (long long)(g.Kp / Z) * ((g.tiles + TB - 1) / TB);
    if (grid_ll > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid_ll), dim3(T), shm, st, x, U2, y, g);
    return hipGetLastError();
}

}  // namespace

// U2: the transformed kernels in the channel-pair layout (launch_wino_kernel_transform_paired), g.Cp / 2 channel
// pairs of g.Kp columns.  g.tb, g.z, g.alpha select the instantiation.
hipError_t launch_wino_fused_rows(const float* x, const float* U2, float* y, const WinoGeom& g, hipStream_t st)
{
    if (g.tiles < 1 || (reinterpret_cast<uintptr_t>(U2) & 15)) return hipErrorInvalidValue;
    if (g.m == 4 && g.tb == 32 && g.z == 64 && g.alpha == 4) return launch_rows_one<4, 1, 2, 4>(x, U2, y, g, st);
    return hipErrorInvalidValue;
}

}  // namespace iolb
