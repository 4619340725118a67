// Direct convolution on the fp32 matrix cores (v_mfma_f32_32x32x2_f32), dataflow of Sec. 5.2.
//
// One workgroup owns an output sub-block of b images * ty rows * tx columns (npix pixels, cut into
// blocks of 32, the last one possibly ragged) by z output channels (a multiple of 32) and keeps its partial sums in accumulator registers
// for the whole channel loop; they are written to HBM once.  The contraction over (c, r, s) runs as an
// implicit GEMM:  acc[z][npix] += W[z][alpha*R*S] * X[alpha*R*S][npix], where X is never materialised:
// each lane reads its pixel's window straight out of the LDS-resident input tile xh * yh.
//
// Per stage of alpha channels (a multiple of 4) the workgroup stages, with LDS-direct loads (no
// registers in between),
//   - the weight slab  [alpha][R*S][z]  from the re-laid-out weights wt[C'][R*S][K'] (C' = C rounded up
//     to whole stages, K' = K rounded up to whole 32-channel blocks, the extra rows and columns zero), whole rows per instruction, 16 bytes per lane;
//   - the input tile   [alpha][b][yh][xh]: the tile of one channel is b*yh*xh contiguous LDS floats, staged in
//     flat chunks of 64 whose lanes each fetch their own element (narrow tile rows share an instruction); tiles
//     with more chunks than a wave keeps offsets for fall back to one instruction per (tile row, 64-column
//     segment, channel).  Elements outside the image are never loaded: the LDS buffers are cleared once and
//     those positions stay zero.
// Two LDS buffers alternate.  The loads of stage s+1 are issued from inside the multiply phase of
// stage s, by the two waves of a SIMD half a stage apart, so that the matrix core always has a wave
// that is multiplying.
//
// Wave layout: waves_m x waves_n waves; a wave owns MBW x NBW blocks of 32 x 32 partial sums.
// Inside one MFMA the two k-slices are fed by lane halves: lanes 0-31 take channel c2, lanes 32-63 take
// channel c2 + alpha/2, so that both halves use the same LDS offset per (r, s).  The LDS reads of step
// j+1 are interleaved between the MFMAs of step j (an MFMA blocks its wave's issue while it runs, so
// a wave must never have a stretch without one).
//
// The kernel is a template over the tensor layout: HWC = false reads x[N][C][H][W] and writes
// y[N][K][P][Q]; HWC = true reads x[N][H][W][C] and writes y[N][P][Q][K] (the layout choice of Table 1,
// Sec. 6.2).  The LDS tile and the multiply phase are the same for both; only the addresses of the
// staging loads and of the final stores differ.  Each layout is instantiated in a source file of its own.
#ifndef IOLB_DIRECT_MFMA_IMPL_H
#define IOLB_DIRECT_MFMA_IMPL_H

#include "kernels.h"
#include "lds_dma.h"

#include <type_traits>

namespace iolb {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// chunks of 64 input-tile elements whose load offsets a wave keeps in registers (flat staging)
constexpr int FLAT_CHUNKS = 8;
template <int MBW, int NBW, int LB, int RR, int SS, bool HWC, bool EVEN>
__global__ void __launch_bounds__(LB, LB <= 256 ? 2 : 1)
direct_mfma_kernel(const float* __restrict__ x, const float* __restrict__ wt, float* __restrict__ y, DirectGeom g)
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

    // The tile's pixels form ceil(npix / 32) blocks, dealt to the waves_n wave columns as evenly as whole
    // blocks allow: the first `extra` columns own NBW blocks, the others NBW - 1 (all NBW when the blocks
    // divide evenly: the EVEN instantiations).  A wave that owns NBW - 1 blocks runs a copy of the channel loop
    // without the last block.  With waves w and
    // w + 4 on one SIMD this keeps the SIMDs within one block of each other.  Pixel slots past the tile in
    // the last block read the tile's last pixel and store nothing.
    int bbase[NBW], pimg[NBW], ppy[NBW], ppx[NBW];
    const int txy = g.tx * g.ty;
    const int npix = g.b * txy;
    const int nblocks_pix = (npix + 31) >> 5;
    const int col_base = nblocks_pix / g.waves_n, col_extra = nblocks_pix % g.waves_n;
    const int my_blocks = col_base + (wn_i < col_extra ? 1 : 0);              // NBW or NBW - 1
    const int first_block = wn_i * col_base + (wn_i < col_extra ? wn_i : col_extra);
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        const int slot = (first_block + nb) * 32 + l32;
        const int pix = slot < npix ? slot : npix - 1;
        const int rem = pix % txy;
        pimg[nb] = pix / txy;
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

    const int gy0 = y0 * g.stride - g.pad, gx0 = x0 * g.stride - g.pad_w;
    const int nwaves = T >> 6;
    const int tile_rows = g.b * g.yh;                       // rows of the input tile per channel
    const int nseg = (g.xh + 63) >> 6;                      // 64-lane segments per tile row
    const float* wslab = wt + k0;                           // row (c*RS + rs) of the slab starts at wslab + row*K

    // Elements of the tile that fall outside the image are zero in every stage: clear the buffers once (two, or
    // the single one of a layer whose channels fit one stage), then only ever load the elements that exist.
    const int nbuffers = g.C <= g.alpha ? 1 : 2;
    for (int i = tid; i < nbuffers * stage_floats; i += T) lds[i] = 0.f;
    __syncthreads();

    // Input-tile staging comes in two forms.
    //  - flat (g.flat): the tile of one channel is halo contiguous LDS floats (rows back to back); chunk
    //    q = 64 consecutive floats of it is one instruction whose lanes each fetch their own element, so
    //    narrow tile rows share an instruction.  A lane's global offset does not depend on the stage, so
    //    the offsets of the (at most FLAT_CHUNKS) chunks a wave owns are computed once; a lane whose
    //    element lies outside the image (or past the tile) never loads.
    //  - by rows: one instruction per (tile row, 64-column segment, channel), the row's base address
    //    wave-uniform, lanes add their column; used when a wave would own more chunks than it has
    //    registers for.
    const int nchunks = (g.halo + 63) >> 6;
    unsigned flat_off[FLAT_CHUNKS];
    if (g.flat) {
#pragma unroll
        for (int j = 0; j < FLAT_CHUNKS; ++j) {
            const int e = (wave + j * nwaves) * 64 + lane;
            flat_off[j] = ~0u;
            if (e < g.halo) {
                const int im = e / (g.yh * g.xh), rem = e % (g.yh * g.xh);
                const int gy = gy0 + rem / g.xh, gx = gx0 + rem % g.xh;
                if (gy >= 0 && gy < g.H && gx >= 0 && gx < g.W)
                    flat_off[j] = HWC ? 4u * (unsigned)(((im * g.H + gy) * g.W + gx) * g.C)
                                      : 4u * (unsigned)(im * g.C * HW + gy * g.W + gx);
            }
        }
    }
    // first (tile row, segment) item of this wave
    const int im_first = wave / (nseg * g.yh);
    const int hy_first = (wave % (nseg * g.yh)) / nseg, seg_first = wave % nseg;

    // Stage c0..c0+alpha-1 into buf.  Weights: alpha*RS rows of z floats, whole rows per instruction.
    // Channels at or beyond C (last stage when alpha does not divide C) are zero rows in wt and are
    // cleared here for the tile.
    auto issue_stage = [&](int c0, float* buf) {
        stage_rows(wslab + (size_t)c0 * RS * g.Kp, g.Kp, g.z >> 2, g.alpha * RS, buf, wave, nwaves, lane);
        float* xbuf = buf + wfloats;
        if (g.flat) {
            const float* cbase = HWC ? x + (size_t)n0 * HW * g.C + c0 : x + ((size_t)n0 * g.C + c0) * HW;
            const int cstep = HWC ? 1 : HW;
            const unsigned dst0 = lds_byte_address(xbuf) + 256u * (unsigned)wave;
#pragma unroll
            for (int j = 0; j < FLAT_CHUNKS; ++j) {
                if (wave + j * nwaves < nchunks && flat_off[j] != ~0u) {
                    const unsigned dst = dst0 + 256u * (unsigned)(j * nwaves);
                    for (int c = 0; c < g.alpha && c0 + c < g.C; ++c)
                        lds_dma_load_4(cbase + (size_t)c * cstep, flat_off[j], dst + 4u * (unsigned)(c * g.halo));
                }
            }
        } else {
            int im = im_first, hy = hy_first, seg = seg_first;
            for (int item = wave; item < tile_rows * nseg; item += nwaves) {
                const int gy = gy0 + hy;
                const int hx = seg * 64 + lane, gx = gx0 + hx;
                if (gy >= 0 && gy < g.H && hx < g.xh && gx >= 0 && gx < g.W) {
                    const unsigned dst = lds_byte_address(xbuf + (im * g.yh + hy) * g.xh + seg * 64);
                    if constexpr (!HWC) {
                        const float* rowp = x + (((size_t)(n0 + im) * g.C + c0) * g.H + gy) * g.W;
                        for (int c = 0; c < g.alpha && c0 + c < g.C; ++c)
                            lds_dma_load_4(rowp + (size_t)c * HW, 4u * (unsigned)gx, dst + 4u * (unsigned)(c * g.halo));
                    } else {
                        // channels innermost: the lanes of a row segment are C floats apart
                        const float* rowp = x + ((size_t)(n0 + im) * g.H + gy) * g.W * g.C + c0;
                        const unsigned off = 4u * (unsigned)gx * (unsigned)g.C;
                        for (int c = 0; c < g.alpha && c0 + c < g.C; ++c)
                            lds_dma_load_4(rowp + c, off, dst + 4u * (unsigned)(c * g.halo));
                    }
                }
                // next item of this wave: advance (im, hy, seg) by nwaves segments
                seg += nwaves;
                while (seg >= nseg) { seg -= nseg; ++hy; }
                while (hy >= g.yh) { hy -= g.yh; ++im; }
            }
        }
        if (c0 + g.alpha > g.C)
            for (int i = (g.C - c0) * g.halo + tid; i < g.alpha * g.halo; i += T) xbuf[i] = 0.f;
    };

    const int nstages = (g.C + g.alpha - 1) / g.alpha;
    const int nsteps = half_c * RS;
    const int step_r = g.xh - (g.S - 1);                          // tile offset increments at a row wrap
    const int step_c = g.halo - (g.R - 1) * g.xh - (g.S - 1);     // ... and at a channel wrap
    // Waves w and w+4 share a SIMD.  Each stages its part of the NEXT stage from inside the multiply
    // phase of the current one, the second group half a stage later than the first, so that while one
    // wave of a SIMD is busy issuing loads the other keeps the matrix core fed.
    const int issue_group = (wave >> 2) & 1;

    // The whole channel loop for a wave that owns NA pixel blocks (NA = NBW, or NBW - 1 for the wave columns
    // that got one block less).  Both versions execute the same barriers.
    auto run_stages = [&](auto na_c) {
        constexpr int NA = decltype(na_c)::value;
        auto interleave_step = [&]() {
            constexpr int MF = MBW * NA, RD = MBW + NA, PAIRS = (RD + 1) / 2;
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
        auto multiply = [&](const float (&am)[MBW], const float (&bm)[NA]) {
#pragma unroll
            for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
                for (int nb = 0; nb < NA; ++nb)
                    acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x2f32(am[mb], bm[nb], acc[mb][nb], 0, 0, 0);
        };

        issue_stage(0, lds);
        for (int s = 0; s < nstages; ++s) {
            lds_dma_wait_all();
            __syncthreads();                                    // stage s has landed; stage s-1 is consumed
            float* cur = lds + (s & 1) * stage_floats;
            float* nxt = lds + ((s + 1) & 1) * stage_floats;
            const bool more = s + 1 < nstages;
            const int c0_next = (s + 1) * g.alpha;

            if constexpr (RR > 0) {
                // Kernel extents known at compile time: the R*S steps of a channel pair are unrolled, so a
                // step costs its LDS reads and a couple of address adds.  A body is two channel pairs (alpha
                // is a multiple of 4), which keeps the two operand register sets in phase.
                constexpr int RSc = RR * SS, BODY = 2 * RSc;
                const int nbodies = half_c >> 1;
                float fa[2][MBW], fb[2][NA];
                auto fetch = [&](int set, int bi, int t) {
                    const int cl = t / RSc, rs = t % RSc, r = rs / SS, sx = rs % SS;
                    const float* wp = cur + abase + ((2 * bi + cl) * RSc + rs) * g.z;
                    const int sc = (2 * bi + cl) * g.halo + r * g.xh;
#pragma unroll
                    for (int mb = 0; mb < MBW; ++mb) fa[set][mb] = wp[mb * 32];
#pragma unroll
                    for (int nb = 0; nb < NA; ++nb) fb[set][nb] = cur[bbase[nb] + sc + sx];
                };
                fetch(0, 0, 0);
                for (int bi = 0; bi < nbodies; ++bi) {
                    const int bnext = (bi + 1 < nbodies) ? bi + 1 : 0;   // after the last body: wrap, read and drop
#pragma unroll
                    for (int t = 0; t < BODY; ++t) {
                        if (t == 0 || t == RSc) {
                            if (more && bi == 0 && issue_group == (t == 0 ? 0 : 1)) issue_stage(c0_next, nxt);
                        }
                        if (t + 1 < BODY) fetch((t + 1) & 1, bi, t + 1);
                        else              fetch(0, bnext, 0);
                        multiply(fa[t & 1], fb[t & 1]);
                        interleave_step();
                    }
                }
            } else {
                // General loop: steps j = (c2, r, s) flattened, two per iteration with two operand register
                // sets (alpha is a multiple of 4, so the count is even).  After the last step the fetch wraps
                // to step 0 (read and dropped).
                const float* wrow = cur + abase;
                int r = 0, sx = 0, xo = 0;              // position of the NEXT step to fetch
                float a[MBW], bv[NA], a1[MBW], b1[NA];
                auto fetch = [&](float (&an)[MBW], float (&bn)[NA], bool last) {
#pragma unroll
                    for (int mb = 0; mb < MBW; ++mb) an[mb] = wrow[mb * 32];
#pragma unroll
                    for (int nb = 0; nb < NA; ++nb) bn[nb] = cur[bbase[nb] + xo];
                    // advance (r, s), the tile offset xo = c2*halo + r*xh + s and the weight row without branches
                    const int wrap_s = (sx + 1 == g.S), wrap_r = wrap_s & (r + 1 == g.R);
                    xo = last ? 0 : xo + (wrap_r ? step_c : (wrap_s ? step_r : 1));
                    wrow = last ? cur + abase : wrow + g.z;
                    sx = wrap_s ? 0 : sx + 1;
                    r = wrap_r ? 0 : r + wrap_s;
                };
                const int issue_at = issue_group ? ((nsteps >> 1) & ~1) : 0;
                fetch(a, bv, false);
#pragma unroll 1
                for (int j = 0; j < nsteps; j += 2) {
                    if (more && j == issue_at) issue_stage(c0_next, nxt);
                    fetch(a1, b1, false);
                    multiply(a, bv);
                    interleave_step();
                    fetch(a, bv, j + 2 >= nsteps);
                    multiply(a1, b1);
                    interleave_step();
                }
            }
        }

    };
    if (EVEN || my_blocks == NBW) run_stages(std::integral_constant<int, NBW>{});
    else if constexpr (!EVEN && NBW > 1) run_stages(std::integral_constant<int, NBW - 1>{});

    // each partial sum is complete: write the block once.  Register i of a 32 x 32 block holds
    // channel 8*(i/4) + 4*half + i%4 of pixel l32.
    const size_t PQ = (size_t)g.P * g.Q;
    // K rounded up to whole 32-channel blocks (Kp) may exceed K: the channels past K are zero columns of wt
    // and are not stored
    const bool ragged_k = g.Kp != g.K;
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
        if (nb >= my_blocks || (first_block + nb) * 32 + l32 >= npix) continue;
        if (y0 + ppy[nb] >= g.P || x0 + ppx[nb] >= g.Q) continue;     // an edge tile's pixels past the image
        if constexpr (!HWC) {
            float* yp = y + ((size_t)(n0 + pimg[nb]) * g.K + k0) * PQ + (size_t)(y0 + ppy[nb]) * g.Q + x0 + ppx[nb];
#pragma unroll
            for (int mb = 0; mb < MBW; ++mb) {
                const int kbase = (wm_i * MBW + mb) * 32 + 4 * half;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int kk = kbase + 8 * (i >> 2) + (i & 3);
                    if (!ragged_k || k0 + kk < g.K) yp[(size_t)kk * PQ] = acc[mb][nb][i];
                }
            }
        } else {
            // channels innermost: a lane's registers 4j..4j+3 are four neighbouring channels, 16 bytes
            float* yp = y + (((size_t)(n0 + pimg[nb]) * g.P + y0 + ppy[nb]) * g.Q + x0 + ppx[nb]) * g.K + k0;
#pragma unroll
            for (int mb = 0; mb < MBW; ++mb) {
                const int kbase = (wm_i * MBW + mb) * 32 + 4 * half;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int kk = kbase + 8 * j;
                    if (!ragged_k) {
                        floatx4 v = {acc[mb][nb][4 * j], acc[mb][nb][4 * j + 1], acc[mb][nb][4 * j + 2], acc[mb][nb][4 * j + 3]};
                        *reinterpret_cast<floatx4*>(yp + kk) = v;
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (k0 + kk + i < g.K) yp[kk + i] = acc[mb][nb][4 * j + i];
                    }
                }
            }
        }
    }
}

template <int MBW, int NBW, int LB, int RR, int SS, bool HWC, bool EVEN>
hipError_t launch_one(const float* x, const float* wt, float* y, const DirectGeom& g,
                      size_t shm, hipStream_t st)
{
    auto kern = direct_mfma_kernel<MBW, NBW, LB, RR, SS, HWC, EVEN>;
    if (shm > 64 * 1024) {
        const hipError_t e = allow_large_lds((const void*)kern);
        if (e != hipSuccess) return e;
    }
    const int grid = g.nbk * g.nbx * g.nby * g.nbn;
    DirectGeom gl = g;
    // flat staging needs every chunk of a wave in its FLAT_CHUNKS registers and 32-bit byte offsets
    const long long nchunks = ((long long)g.halo + 63) / 64, nwaves = g.threads / 64;
    const long long span = 4LL * g.b * g.C * g.H * g.W;
    gl.flat = (nchunks + nwaves - 1) / nwaves <= FLAT_CHUNKS && span < (1LL << 32);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(g.threads), shm, st, x, wt, y, gl);
    return hipGetLastError();
}

template <bool HWC>
hipError_t launch_direct_mfma_layout(const float* x, const float* wt, float* y, const DirectGeom& g, hipStream_t st)
{
    const int npix = g.b * g.tx * g.ty;
    if (g.z % 32 || (g.alpha & 3) || g.threads != 64 * g.waves_m * g.waves_n) return hipErrorInvalidValue;
    const int MB = g.z / 32, NB = (npix + 31) / 32;          // a ragged last block is masked in the kernel
    if (MB % g.waves_m || g.waves_n > NB) return hipErrorInvalidValue;
    const int mbw = MB / g.waves_m, nbw = (NB + g.waves_n - 1) / g.waves_n;
    const bool even = NB % g.waves_n == 0;                   // every wave column owns nbw blocks
    const size_t stage = ((size_t)g.alpha * ((size_t)g.R * g.S * g.z + g.halo) + 3) & ~(size_t)3;
    const size_t shm = (g.C <= g.alpha ? 1 : 2) * stage * sizeof(float);      // a single stage needs one buffer
    if (shm > 160 * 1024) return hipErrorInvalidValue;
    // the register file of a compute unit holds 131072 lane-registers: a workgroup of T threads gets
    // 131072 / T per lane, of which 16 * mbw * nbw are partial sums
    if (16 * mbw * nbw + 64 > 131072 / g.threads) return hipErrorInvalidValue;
#define IOLB_CASE(M_, N_)                                                                              \
    if (mbw == M_ && nbw == N_) {                                                                      \
        if (g.R == 3 && g.S == 3) {                                                                    \
            if (g.threads <= 256) return even ? launch_one<M_, N_, 256, 3, 3, HWC, true>(x, wt, y, g, shm, st) : launch_one<M_, N_, 256, 3, 3, HWC, false>(x, wt, y, g, shm, st);          \
            if (g.threads <= 512) return even ? launch_one<M_, N_, 512, 3, 3, HWC, true>(x, wt, y, g, shm, st) : launch_one<M_, N_, 512, 3, 3, HWC, false>(x, wt, y, g, shm, st);          \
            if constexpr (M_ * N_ <= 4) return even ? launch_one<M_, N_, 1024, 3, 3, HWC, true>(x, wt, y, g, shm, st) : launch_one<M_, N_, 1024, 3, 3, HWC, false>(x, wt, y, g, shm, st);   \
        } else {                                                                                       \
            if (g.threads <= 256) return even ? launch_one<M_, N_, 256, 0, 0, HWC, true>(x, wt, y, g, shm, st) : launch_one<M_, N_, 256, 0, 0, HWC, false>(x, wt, y, g, shm, st);          \
            if (g.threads <= 512) return even ? launch_one<M_, N_, 512, 0, 0, HWC, true>(x, wt, y, g, shm, st) : launch_one<M_, N_, 512, 0, 0, HWC, false>(x, wt, y, g, shm, st);          \
            if constexpr (M_ * N_ <= 4) return even ? launch_one<M_, N_, 1024, 0, 0, HWC, true>(x, wt, y, g, shm, st) : launch_one<M_, N_, 1024, 0, 0, HWC, false>(x, wt, y, g, shm, st);   \
        }                                                                                              \
    }
    IOLB_CASE(1, 1) IOLB_CASE(1, 2) IOLB_CASE(1, 3) IOLB_CASE(1, 4)
    IOLB_CASE(1, 5) IOLB_CASE(1, 6) IOLB_CASE(1, 7) IOLB_CASE(1, 8)
    IOLB_CASE(2, 1) IOLB_CASE(2, 2) IOLB_CASE(2, 3) IOLB_CASE(2, 4)
#undef IOLB_CASE
    return hipErrorInvalidValue;
}


}  // namespace

}  // namespace iolb

#endif
