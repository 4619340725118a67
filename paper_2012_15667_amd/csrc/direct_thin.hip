// Direct convolution for thin layers (a handful of input channels, 3 x 3 kernels, stride 1): the dataflow of
// Sec. 5.2 with the on-chip block held in registers.
//
// One lane owns TW neighbouring output pixels of a row and every output channel.  It loads the 3 x (TW + 2) input
// window of all C channels once and keeps it in registers; then it walks over the output channels: the 9 C
// kernel elements of an output channel are the same for every lane and are read through the scalar unit (one
// contiguous row per output channel, 16 floats at a time), 9 C TW fused multiply-adds follow, and the TW results
// are stored (one 16-byte store when the row allows).  Inputs are read once, outputs written once, the kernels
// come from the scalar cache: the layer moves its compulsory bytes, and the stores of one wave run beside the
// arithmetic of the others -- which the matrix-core kernel, where a workgroup multiplies for one short stage and
// then stores for much longer, cannot arrange on such a layer.  The contraction over 9 C values is too thin for
// the matrix cores; it runs as plain fp32 FMAs.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "kernels.h"

namespace iolb {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Row length of the kernel elements of one output channel, [c][r][s], rounded up to whole 16-float pieces.
constexpr int thin_row(int c) { return (9 * c + 15) / 16 * 16; }

template <int CC, int TW, bool VEC>
__global__ void __launch_bounds__(256)
direct_thin_kernel(const float* __restrict__ x, const float* __restrict__ wk, float* __restrict__ y, DirectGeom g, int kc)
{
    constexpr int ROW = thin_row(CC), XW = TW + 2;
    const int groups = (g.Q + TW - 1) / TW;                       // lanes per output row
    const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
    if (t >= (long long)g.N * g.P * groups) return;               // no barriers below
    const int qg = (int)(t % groups), p = (int)((t / groups) % g.P), img = (int)(t / ((long long)groups * g.P));
    const int q0 = qg * TW;
    const int h0 = p - g.pad, w0 = q0 - g.pad_w;

    // every load is issued, from an address clamped into the image, and zeroed afterwards if it lies outside: no
    // branches, so the loads of a window are in flight together
    float d[CC][3][XW];
#pragma unroll
    for (int c = 0; c < CC; ++c) {
        const float* xp = x + ((size_t)img * CC + c) * g.H * g.W;
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int j = 0; j < XW; ++j) {
                const int h = h0 + i, ww = w0 + j;
                const int hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h), wc = ww < 0 ? 0 : (ww >= g.W ? g.W - 1 : ww);
                d[c][i][j] = xp[(size_t)hc * g.W + wc];
            }
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int j = 0; j < XW; ++j) {
                const int h = h0 + i, ww = w0 + j;
                if (!(h >= 0 && h < g.H && ww >= 0 && ww < g.W)) d[c][i][j] = 0.f;
            }
    }

    const size_t yplane = (size_t)g.P * g.Q;
    float* yp = y + (size_t)img * g.K * yplane + (size_t)p * g.Q + q0;
    // blockIdx.y selects kc output channels: their rows stay in the scalar cache while the workgroups of the same
    // channel group, which are dispatched together, walk over them
    const int k_begin = blockIdx.y * kc, k_end = k_begin + kc < g.K ? k_begin + kc : g.K;
#pragma unroll 4
    for (int k = k_begin; k < k_end; ++k) {
        const float* uk = wk + (size_t)k * ROW;                   // the same for every lane: scalar loads
        float o[TW];
#pragma unroll
        for (int q = 0; q < 9 * CC; q += 16) {
            const floatx16 u = *reinterpret_cast<const floatx16*>(uk + q);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int idx = q + e;
                if (idx < 9 * CC) {
                    const int c = idx / 9, r = (idx % 9) / 3, s = idx % 3;
#pragma unroll
                    for (int j = 0; j < TW; ++j)
                        o[j] = idx == 0 ? u[e] * d[0][0][j] : __builtin_fmaf(u[e], d[c][r][j + s], o[j]);
                }
            }
        }
        float* yk = yp + (size_t)k * yplane;
        if constexpr (VEC) {
            typedef float vec __attribute__((ext_vector_type(TW)));
            vec v;
#pragma unroll
            for (int j = 0; j < TW; ++j) v[j] = o[j];
            __builtin_nontemporal_store(v, reinterpret_cast<vec*>(yk));      // written once, not read again here
        } else {
#pragma unroll
            for (int j = 0; j < TW; ++j)
                if (q0 + j < g.Q) yk[j] = o[j];
        }
    }
}

// wk[k][i] = w[k][i] for i < 9 C (w is [K][C][3][3]: the 9 C elements of a kernel are contiguous), 0 up to the row end
__global__ void __launch_bounds__(256)
thin_rows_kernel(const float* __restrict__ w, float* __restrict__ wk, int K, int crs, int row)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= K * row) return;
    const int k = idx / row, q = idx % row;
    wk[idx] = q < crs ? w[(size_t)k * crs + q] : 0.f;
}

template <int CC>
hipError_t launch_thin_c(const float* x, const float* wk, float* y, const DirectGeom& g, hipStream_t st)
{
    // output channels per workgroup: as many rows as fit in 12 KB of the 16 KB scalar cache
    constexpr int row_bytes = 4 * thin_row(CC);
    const int kc = 12288 / row_bytes >= g.K ? g.K : 12288 / row_bytes / 8 * 8;
    const bool vec = g.Q % 4 == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0;
    const int tw = vec ? 4 : 1;
    const long long lanes = (long long)g.N * g.P * ((g.Q + tw - 1) / tw);
    const long long blocks = (lanes + 255) / 256;
    const dim3 grid((unsigned)blocks, (g.K + kc - 1) / kc);
    if (blocks > 0x7fffffffLL || grid.y > 65535) return hipErrorInvalidValue;
    if (vec) hipLaunchKernelGGL((direct_thin_kernel<CC, 4, true>), grid, dim3(256), 0, st, x, wk, y, g, kc);
    else     hipLaunchKernelGGL((direct_thin_kernel<CC, 1, false>), grid, dim3(256), 0, st, x, wk, y, g, kc);
    return hipGetLastError();
}

}  // namespace

int direct_thin_row(int C) { return thin_row(C); }

hipError_t launch_direct_thin_rows(const float* w, float* wk, int K, int C, hipStream_t st)
{
    const int row = thin_row(C);
    if (K < 1 || C < 1 || (int64_t)K * row >= (1LL << 31)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(thin_rows_kernel, dim3((K * row + 255) / 256), dim3(256), 0, st, w, wk, K, 9 * C, row);
    return hipGetLastError();
}

// wk: K rows of direct_thin_row(C) floats, 64-byte aligned; x, y plain NCHW tensors; 3 x 3 kernels, stride 1, C <= 4.
hipError_t launch_direct_thin(const float* x, const float* wk, float* y, const DirectGeom& g, hipStream_t st)
{
    if (g.R != 3 || g.S != 3 || g.stride != 1 || g.hwc || g.w_transposed) return hipErrorInvalidValue;
    if (g.P != g.H + 2 * g.pad - 2 || g.Q != g.W + 2 * g.pad_w - 2 || g.P < 1 || g.Q < 1) return hipErrorInvalidValue;
    if (reinterpret_cast<uintptr_t>(wk) & 63) return hipErrorInvalidValue;
    switch (g.C) {
    case 1: return launch_thin_c<1>(x, wk, y, g, st);
    case 2: return launch_thin_c<2>(x, wk, y, g, st);
    case 3: return launch_thin_c<3>(x, wk, y, g, st);
    case 4: return launch_thin_c<4>(x, wk, y, g, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace iolb
