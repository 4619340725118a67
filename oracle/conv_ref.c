/*
 * TEST INFRASTRUCTURE ONLY -- the CPU oracle for the forward 2-D convolution layer.
 *
 * This file is a plain, slow, obviously-correct statement of what a convolution
 * layer computes (paper Sec. 2.2 "Direct Convolution": every output is the inner
 * product of one kernel tensor with one sliding window of the input, adjacent
 * windows being `stride` positions apart; Sec. 4.2 describes the same thing as a
 * two-step DAG: all products, then one summation tree per output).
 *
 * It is compiled with the host C compiler only and shares no code with the GPU
 * library.  Only tests, the smoke check and the CPU-baseline leg of the benchmark
 * may call it.
 *
 * Conventions fixed here (the paper leaves them open):
 *   - cross-correlation, no kernel flip;
 *   - zero padding of `pad` positions on every side;
 *   - output extent  P = floor((H + 2*pad - R)/stride) + 1, Q likewise from W and S;
 *   - a batch of N independent images shares one set of K kernels;
 *   - x is [N][C][H][W], w is [K][C][R][S], y is [N][K][P][Q], all dense, row-major;
 *   - fp32 inputs are widened to fp64, one fp64 accumulator per output, summation
 *     in (c, r, s) ascending order, result kept in fp64.
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double one_output(const float *x, const float *w,
                         int C, int H, int W, int R, int S, int stride, int pad,
                         int n, int k, int p, int q)
{
    double acc = 0.0;
    for (int c = 0; c < C; ++c) {
        for (int r = 0; r < R; ++r) {
            for (int s = 0; s < S; ++s) {
                int h  = p * stride + r - pad;
                int wq = q * stride + s - pad;
                if (h < 0 || h >= H || wq < 0 || wq >= W) continue;   /* zero padding */
                double xv = (double)x[(((size_t)n * C + c) * H + h) * W + wq];
                double wv = (double)w[(((size_t)k * C + c) * R + r) * S + s];
                acc += xv * wv;
            }
        }
    }
    return acc;
}

/* Full layer.  Returns the number of threads the loop nest ran on, or -1 on bad arguments. */
int conv_ref_f64(const float *x, const float *w, double *y,
                 int N, int C, int H, int W, int K, int R, int S, int stride, int pad)
{
    if (!x || !w || !y || N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1 ||
        stride < 1 || pad < 0) return -1;
    if (H + 2 * pad < R || W + 2 * pad < S) return -1;
    const int P = (H + 2 * pad - R) / stride + 1;
    const int Q = (W + 2 * pad - S) / stride + 1;
    int threads = 1;
#ifdef _OPENMP
    threads = omp_get_max_threads();
#pragma omp parallel for collapse(2) schedule(static)
#endif
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            for (int p = 0; p < P; ++p) {
                for (int q = 0; q < Q; ++q) {
                    y[(((size_t)n * K + k) * P + p) * Q + q] =
                        one_output(x, w, C, H, W, R, S, stride, pad, n, k, p, q);
                }
            }
        }
    }
    return threads;
}

/* The same definition evaluated only at `count` chosen outputs; idx holds (n,k,p,q) quadruples.
 * Used to check full-size layers on a sample.  Returns 0, or -1 on bad arguments. */
int conv_ref_points_f64(const float *x, const float *w, const int32_t *idx, int64_t count, double *out,
                        int N, int C, int H, int W, int K, int R, int S, int stride, int pad)
{
    if (!x || !w || !idx || !out || count < 0 || N < 1 || C < 1 || H < 1 || W < 1 || K < 1 ||
        R < 1 || S < 1 || stride < 1 || pad < 0) return -1;
    if (H + 2 * pad < R || W + 2 * pad < S) return -1;
    const int P = (H + 2 * pad - R) / stride + 1;
    const int Q = (W + 2 * pad - S) / stride + 1;
    for (int64_t i = 0; i < count; ++i) {
        int n = idx[4 * i], k = idx[4 * i + 1], p = idx[4 * i + 2], q = idx[4 * i + 3];
        if (n < 0 || n >= N || k < 0 || k >= K || p < 0 || p >= P || q < 0 || q >= Q) return -1;
    }
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int64_t i = 0; i < count; ++i) {
        out[i] = one_output(x, w, C, H, W, R, S, stride, pad,
                            idx[4 * i], idx[4 * i + 1], idx[4 * i + 2], idx[4 * i + 3]);
    }
    return 0;
}
