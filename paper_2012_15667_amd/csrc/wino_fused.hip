// Winograd F(m x m, 3 x 3) for thin layers (a handful of input channels): the four steps of Sec. 4.3 in one
// kernel, the dataflow of Sec. 5.3 with the on-chip block held in registers.
//
// One lane owns one sub-domain.  It loads the (m+2) x (m+2) input windows of all C channels, transforms them
// (step 1a) and keeps the C * (m+2)^2 transformed values in registers for the rest of the kernel.  Then it
// walks over the output channels: the element-wise products and the channel sum (steps 2 and 3) are C fused
// multiply-adds per transformed position, whose kernel-side factor is the same for every lane and is read
// through the scalar unit (the C * (m+2)^2 factors of one output channel form one contiguous row, fetched 16
// at a time); the output transform (step 4) follows at once and the m x m results are stored.  Neither the transformed inputs nor the channel-summation temporaries ever leave
// the registers, so the layer moves its compulsory bytes only -- against a round trip of (m+2)^2 / m^2 times
// the output tensor for the temporaries of the unfused path, which is what bounds that path on such layers.
// The contraction over C is too thin for the matrix cores; it runs as plain fp32 FMAs.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "kernels.h"
#include "wino_transform.h"

namespace iolb {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Row length of the kernel-side factors: the C * (m+2)^2 values of one output channel, [xi][c], rounded up
// to whole 16-float pieces (one scalar load each).
constexpr int fused_row(int m, int c) { return ((m + 2) * (m + 2) * c + 15) / 16 * 16; }

template <int M, int CC, bool VEC>
__global__ void __launch_bounds__(256)
wino_fused_kernel(const float* __restrict__ x, const float* __restrict__ Uk, float* __restrict__ y, WinoGeom g, int kc)
{
    constexpr int n = Mats<M>::n;
    constexpr int PC = n * n * CC, ROW = fused_row(M, CC);
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= g.tiles) return;                                   // no barriers below
    const int tj = t % g.tw, ti = (t / g.tw) % g.th, img = t / (g.tw * g.th);
    const int h0 = ti * M - g.pad, w0 = tj * M - g.pad;

    float v[CC][n][n];
    static_for<CC>([&](auto c) {
        const float* xp = x + ((size_t)img * CC + c) * g.H * g.W;
        float d[n][n], tmp[n][n];
        // every load is issued, from an address clamped into the image, and zeroed afterwards if it lies
        // outside: no branches, so the loads of a window are in flight together
#pragma unroll
        for (int i = 0; i < n; ++i)
#pragma unroll
            for (int j = 0; j < n; ++j) {
                const int h = h0 + i, ww = w0 + j;
                const int hc = h < 0 ? 0 : (h >= g.H ? g.H - 1 : h), wc = ww < 0 ? 0 : (ww >= g.W ? g.W - 1 : ww);
                d[i][j] = xp[(size_t)hc * g.W + wc];
            }
#pragma unroll
        for (int i = 0; i < n; ++i)
#pragma unroll
            for (int j = 0; j < n; ++j) {
                const int h = h0 + i, ww = w0 + j;
                if (!(h >= 0 && h < g.H && ww >= 0 && ww < g.W)) d[i][j] = 0.f;
            }
        left_mul<M, UseB, n, n, n>(d, tmp);
        right_mul_t<M, UseB, n, n, n>(tmp, v[c]);
    });

    const size_t yplane = (size_t)g.P * g.Q;
    float* yp = y + (size_t)img * g.K * yplane + (size_t)(ti * M) * g.Q + tj * M;
    // blockIdx.y selects kc output channels: their factor rows stay in the scalar cache while the
    // workgroups of the same channel group, which are dispatched together, walk over them
    const int k_begin = blockIdx.y * kc, k_end = k_begin + kc < g.K ? k_begin + kc : g.K;
#pragma unroll 2
    for (int k = k_begin; k < k_end; ++k) {
        const float* uk = Uk + (size_t)k * ROW;                 // the same for every lane: scalar loads
        float mm[n][n];
#pragma unroll
        for (int q = 0; q < PC; q += 16) {
            const floatx16 u = *reinterpret_cast<const floatx16*>(uk + q);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int idx = q + e;
                if (idx < PC) {
                    const int xi = idx / CC, c = idx % CC, i = xi / n, j = xi % n;
                    mm[i][j] = c == 0 ? u[e] * v[0][i][j] : __builtin_fmaf(u[e], v[c][i][j], mm[i][j]);
                }
            }
        }
        float tmp[M][n], o[M][M];
        left_mul<M, UseA, M, n, n>(mm, tmp);
        right_mul_t<M, UseA, M, n, M>(tmp, o);
        float* yk = yp + (size_t)k * yplane;
#pragma unroll
        for (int i = 0; i < M; ++i) {
            const int h = ti * M + i;
            if constexpr (VEC) {
                typedef float vec __attribute__((ext_vector_type(M)));
                vec q;
#pragma unroll
                for (int j = 0; j < M; ++j) q[j] = o[i][j];
                if (h < g.P) __builtin_nontemporal_store(q, reinterpret_cast<vec*>(yk + (size_t)i * g.Q));
            } else {
#pragma unroll
                for (int j = 0; j < M; ++j)
                    if (h < g.P && tj * M + j < g.Q) yk[(size_t)i * g.Q + j] = o[i][j];
            }
        }
    }
}

// Uk[k][xi * C + c] = U[xi][c][k] for k < K: the row-per-output-channel form of kernels that were
// transformed into the plane-major layout beforehand.
__global__ void __launch_bounds__(256)
fused_relayout_kernel(const float* __restrict__ U, float* __restrict__ Uk, int C, int CpU, int Kp, int K, int pc, int row)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= K * row) return;
    const int k = idx / row, q = idx % row;
    Uk[idx] = q < pc ? U[((size_t)(q / C) * CpU + q % C) * Kp + k] : 0.f;
}

template <int M, int CC>
hipError_t launch_fused_mc(const float* x, const float* U, float* y, const WinoGeom& g, hipStream_t st)
{
    // output channels per workgroup: as many factor rows as fit in 12 KB of the 16 KB scalar cache
    constexpr int row_bytes = 4 * fused_row(M, CC);
    const int kc = 12288 / row_bytes >= g.K ? g.K : 12288 / row_bytes / 8 * 8;
    const dim3 grid((g.tiles + 255) / 256, (g.K + kc - 1) / kc);
    if (grid.y > 65535) return hipErrorInvalidValue;
    constexpr bool can_vec = M == 2 || M == 4;
    const bool vec = can_vec && g.Q % M == 0 && (reinterpret_cast<uintptr_t>(y) & (4 * M - 1)) == 0;
    if constexpr (can_vec) {
        if (vec) {
            hipLaunchKernelGGL((wino_fused_kernel<M, CC, true>), grid, dim3(256), 0, st, x, U, y, g, kc);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((wino_fused_kernel<M, CC, false>), grid, dim3(256), 0, st, x, U, y, g, kc);
    return hipGetLastError();
}

template <int M>
hipError_t launch_fused_m(const float* x, const float* U, float* y, const WinoGeom& g, hipStream_t st)
{
    constexpr int n2 = (M + 2) * (M + 2);
    switch (g.C) {
    case 1: return launch_fused_mc<M, 1>(x, U, y, g, st);
    case 2: if constexpr (2 * n2 <= 128) return launch_fused_mc<M, 2>(x, U, y, g, st); break;
    case 3: if constexpr (3 * n2 <= 128) return launch_fused_mc<M, 3>(x, U, y, g, st); break;
    case 4: if constexpr (4 * n2 <= 128) return launch_fused_mc<M, 4>(x, U, y, g, st); break;
    default: break;
    }
    return hipErrorInvalidValue;
}

}  // namespace

int wino_fused_row(int m, int C) { return fused_row(m, C); }

hipError_t launch_wino_fused_relayout(const float* U, float* Uk, const WinoGeom& g, hipStream_t st)
{
    const int pc = (g.m + 2) * (g.m + 2) * g.C, row = fused_row(g.m, g.C);
    if (g.CpU < g.C || (int64_t)g.K * row >= (1LL << 31)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(fused_relayout_kernel, dim3((g.K * row + 255) / 256), dim3(256), 0, st, U, Uk, g.C, g.CpU, g.Kp, g.K, pc, row);
    return hipGetLastError();
}

// Uk: K rows of wino_fused_row(m, C) floats, Uk[k][xi * C + c] = (L g_{k,c} L^T)[xi], 64-byte aligned;
// x, y plain NCHW tensors.  C <= 4 and C * (m+2)^2 <= 128.
hipError_t launch_wino_fused(const float* x, const float* U, float* y, const WinoGeom& g, hipStream_t st)
{
    if (g.tiles < 1 || (reinterpret_cast<uintptr_t>(U) & 63)) return hipErrorInvalidValue;
    switch (g.m) {
    case 2: return launch_fused_m<2>(x, U, y, g, st);
    case 3: return launch_fused_m<3>(x, U, y, g, st);
    case 4: return launch_fused_m<4>(x, U, y, g, st);
    case 6: return launch_fused_m<6>(x, U, y, g, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace iolb
