/*
 * iolbconv -- forward 2-D convolution for AMD MI355X (gfx950), tiled by the red-blue-pebble
 * I/O lower bound of "I/O Lower Bounds for Auto-tuning of Convolutions in CNNs".
 *
 * C ABI.  Every tensor pointer is a DEVICE pointer to dense fp32 data owned by the caller; the
 * library never frees or keeps them.  All entry points return 0 on success or a negative
 * IOLB_E* code; no exception crosses this boundary and nothing aborts.  Arguments are checked
 * before anything is launched, so a call that fails validation writes nothing.
 *
 * Work is enqueued on the stream given to iolb_set_stream (the null stream by default; the setting is per host
 * thread) and the calls return without waiting for it.  Thread-compatible with one stream per host thread: the
 * library keeps one workspace per (GPU, stream), so calls on different streams do not share scratch memory;
 * calls on one stream are ordered by the stream.  A call that does not have to grow its stream's workspace
 * enqueues kernels only (no allocation, no memset, no synchronisation), so after one eager call for the same
 * layer on the same stream it can be recorded by a stream capture and replayed as a graph.  A workspace that
 * has to grow is replaced, never freed before iolb_release_workspace, so kernels in flight and graphs captured
 * earlier keep valid addresses; iolb_release_workspace invalidates such graphs.
 *
 * Symbols (paper -> here): W_in,H_in,C_in -> W,H,C;  C_out -> K;  W_ker,H_ker -> S,R;
 * W_out,H_out -> Q,P;  mu -> stride;  e -> m.  A batch of N images shares the K kernels.
 */
#ifndef IOLBCONV_H
#define IOLBCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define IOLB_OK            0
#define IOLB_EINVAL       -1   /* null pointer, non-positive extent, stride < 1, pad < 0, empty output */
#define IOLB_EUNSUPPORTED -2   /* Winograd m outside {2,3,4,6}; algo or layout outside its enum */
#define IOLB_ENOTILE      -3   /* no tile fits the LDS / register budgets */
#define IOLB_EWORKSPACE   -4   /* workspace missing or too small */
#define IOLB_EHIP         -5   /* a HIP runtime call or launch failed; see iolb_last_hip_error */

enum { IOLB_DIRECT = 0, IOLB_WINO_F2 = 1, IOLB_WINO_F4 = 2, IOLB_WINO_F3 = 3, IOLB_WINO_F6 = 4 };
enum { IOLB_PATH_FMA = 0, IOLB_PATH_MFMA = 1, IOLB_PATH_FUSED = 2, IOLB_PATH_POINT = 3 };
/* FUSED: Winograd only, all four steps in one matrix-core kernel (Sec. 5.3).  POINT: direct convolution with
 * R = S = 1, no padding, channels-outermost tensors only: the dataflow of Sec. 5.2 on the output plane taken as
 * one row of P * Q pixels (without a kernel window the pixels do not interact). */
enum { IOLB_LAYOUT_CHW = 0, IOLB_LAYOUT_HWC = 1, IOLB_LAYOUT_CWH = 2 };   /* per image: channels outermost, channels
                                                                           innermost, channels outermost with W before H */

/* A convolution layer (Sec. 2.2).  Output extents are P = floor((H+2 pad-R)/stride)+1 and
 * Q = floor((W+2 pad-S)/stride)+1.  For the Winograd algos R = S = 3 and stride = 1. */
typedef struct iolb_shape {
    int32_t N, C, H, W, K, R, S, stride, pad;
    int32_t algo;               /* IOLB_DIRECT or IOLB_WINO_F2 / _F3 / _F4 / _F6 (m = 2, 3, 4, 6) */
} iolb_shape;

/* A tile configuration: the output sub-block x * y * z of Sec. 5.2 (x along W_out, y along
 * H_out, z along C_out) taken over b images, the channels per stage alpha, and the thread
 * decomposition (Table 1 of Sec. 6.2: tile sizes and thread numbers).
 * For the Winograd algos the block is a strip of x/m sub-domains of m x m outputs (b = 1,
 * y = m) of one transformed plane.  For IOLB_PATH_POINT the block is x consecutive pixels of the image
 * taken as one row of P * Q pixels (b = 1, y = 1; a block may run on into the next image) by z output
 * channels.  All fields are exact integers. */
typedef struct iolb_tile_config {
    int32_t b, x, y, z;
    int32_t alpha;               /* input channels staged per step of the channel loop */
    int32_t threads;             /* workgroup size */
    int32_t waves_m, waves_n;    /* MFMA path: wave grid over (z, pixels); FMA path: channel groups, 1 */
    int32_t path;                /* IOLB_PATH_FMA, _MFMA, _FUSED or _POINT */
    int32_t wt_mode;             /* 0: raw R*S weights staged; 1: pre-transformed (m+2)^2 weights; 2: thin direct
                                    layers (3 x 3, stride 1, C <= 4, channels-outermost tensors): one lane per x / 256
                                    neighbouring pixels of a row and all z = K channels, kernels through the scalar unit */
    int32_t lds_bytes_used;      /* staging bytes the tile needs */
    int32_t acc_regs_per_thread; /* partial sums held per lane */
    int64_t q_read_elems;        /* modelled elements read by all workgroups (exact form of the
                                    reading volume of Sec. 5.2 / 5.3 for this tile) */
    int64_t q_write_elems;       /* N*K*P*Q: every output written once */
} iolb_tile_config;

/* Figures of the lower-bound theory for one layer at fast-memory size S_f (in elements). */
typedef struct iolb_bounds_out {
    int32_t P, Q;
    int64_t vertices;            /* internal+output vertices of the DAG: Sec. 4.2 second lemma
                                    (direct); per-step counts of the Sec. 4.3 lemma (Winograd) */
    int64_t compulsory_elems;    /* N*C*H*W + K*C*R*S + N*K*P*Q (Sec. 3.1: each input loaded and
                                    each output stored at least once) */
    int64_t q_write_elems;
    double  t_bound_2s;          /* T(2 S_f): Sec. 4.2 third lemma / Sec. 4.3 T lemma */
    double  q_lower_lead;        /* leading term printed in the theorems of Sec. 4.2 / 4.3 */
    double  q_lower_explicit;    /* S_f (|V|/T(2 S_f) - 1), the general theorem of Sec. 4.1 */
    double  q_dataflow;          /* total volume of the near-optimal dataflow, Sec. 5.2 / 5.3, N_p = 1 */
} iolb_bounds_out;

/* Direct convolution (Sec. 2.2, dataflow of Sec. 5.2).
 *   y[n,k,p,q] = sum_{c,r,s} xpad[n,c,p*stride+r-pad,q*stride+s-pad] * w[k,c,r,s]
 * x: [N][C][H][W], w: [K][C][R][S], y: [N][K][P][Q]; cross-correlation, zero padding.
 * y is fully overwritten; x and y must not overlap.  The tile comes from iolb_tune with the
 * default budgets.  May grow the stream's workspace in the library (one allocation, kept). */
int conv_direct(const float* x, const float* w, float* y,
                int N, int C, int H, int W, int K, int R, int S, int stride, int pad);

/* Same, with the tile given by the caller (for sweeps).  cfg must be one that iolb_tune or
 * iolb_enumerate produced for this shape; IOLB_EINVAL otherwise. */
int conv_direct_cfg(const float* x, const float* w, float* y,
                    int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                    const iolb_tile_config* cfg);

/* Direct convolution with the tensor layout as a parameter (the layout entry of the searching
 * domain, Table 1 of Sec. 6.2).  IOLB_LAYOUT_CHW: as conv_direct.  IOLB_LAYOUT_HWC:
 * x: [N][H][W][C], y: [N][P][Q][K].  IOLB_LAYOUT_CWH: x: [N][C][W][H], y: [N][K][Q][P] (the
 * transposed image: computed as the CHW convolution of the W x H image with the kernels
 * transposed, so tiles are those of that transposed layer).  w is [K][C][R][S] for all.  cfg may be NULL (the tuned
 * tile is used; tiles do not depend on the layout, except that IOLB_PATH_POINT tiles and the thin-layer tiles
 * (wt_mode 2) exist for IOLB_LAYOUT_CHW only: IOLB_EINVAL with another layout; with cfg NULL the best other tile is used).  Other layout values: IOLB_EUNSUPPORTED. */
int conv_direct_layout(const float* x, const float* w, float* y,
                       int N, int C, int H, int W, int K, int R, int S, int stride, int pad,
                       int layout, const iolb_tile_config* cfg);

/* conv_direct for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, layouts and result (bit for bit) as conv_direct, but
 * the re-laid-out weights go into a fixed array inside the library instead of the grown workspace: the call
 * makes no hipMalloc / hipFree and no allocating library call, and enqueues kernels only.
 * Limit: K rounded up to 32, times C rounded up to whole stages (at most 16 extra channels), times R * S must
 * not exceed conv_direct_noalloc_max_weight_floats() = 4194304 floats (16 MiB, held by every GPU the library
 * has run this call on until the process ends); beyond it the call returns IOLB_EWORKSPACE and launches
 * nothing.  All calls on one GPU share that array: calls that overlap on one GPU (two streams) race, and a
 * captured graph must not replay concurrently with another call of this entry point on the same GPU. */
int conv_direct_noalloc(const float* x, const float* w, float* y,
                        int N, int C, int H, int W, int K, int R, int S, int stride, int pad);
size_t conv_direct_noalloc_max_weight_floats(void);

/* conv_direct with its own padding per axis: pad_h rows of zeros above and below, pad_w columns left and
 * right (the 1 x 7 / 7 x 1 factorised kernels of Inception-v3 pad one axis only); P and Q follow from
 * pad_h and pad_w.  NCHW tensors, tuned tile. */
int conv_direct_pad2(const float* x, const float* w, float* y,
                     int N, int C, int H, int W, int K, int R, int S, int stride, int pad_h, int pad_w);

/* Winograd F(m x m, 3 x 3) convolution (Sec. 2.3; four steps of Sec. 4.3), R = S = 3,
 * stride 1, pad 1 (P = H, Q = W), m in {2, 3, 4, 6} (Sec. 2.3 names e = 2 and e = 3; larger m
 * trades more rounding error for fewer multiplications).  Same layouts as conv_direct.  The transformed
 * kernels, inputs and products live in the library's device workspace, grown on demand.
 * Thin layers (C <= 4 and C * (m+2)^2 <= 128; the tuned tile then has path == IOLB_PATH_FMA) run the
 * fused dataflow of Sec. 5.3 as one kernel: transformed inputs and channel sums stay in registers, the
 * workspace holds the transformed kernels only. */
int conv_winograd(const float* x, const float* w, float* y,
                  int N, int C, int H, int W, int K, int m);

/* conv_winograd with `pad` zeros on every side instead of one (pad >= 0, H + 2 pad >= 3, W + 2 pad >= 3):
 * y is [N][K][H + 2 pad - 2][W + 2 pad - 2].  Sub-domain (i, j) reads the (m+2) x (m+2) window whose corner is
 * (i m - pad, j m - pad).  Library workspace, tuned tile. */
int conv_winograd_pad(const float* x, const float* w, float* y,
                      int N, int C, int H, int W, int K, int m, int pad);

/* Bytes of workspace conv_winograd_ws needs for this layer (0 on invalid arguments). */
size_t conv_winograd_workspace_bytes(int N, int C, int H, int W, int K, int m);

/* conv_winograd with a caller-owned device workspace of at least that many bytes, 256-byte
 * aligned.  cfg may be NULL (the tuned tile is used). */
int conv_winograd_ws(const float* x, const float* w, float* y,
                     int N, int C, int H, int W, int K, int m,
                     void* workspace, size_t workspace_bytes, const iolb_tile_config* cfg);

/* Kernels transformed once, used by many calls (inference: the weights do not change).
 * conv_winograd_kernel_bytes: size of the transformed-kernel buffer for C x K kernels of
 * F(m x m, 3 x 3) (0 on invalid arguments).  conv_winograd_transform_kernels: writes
 * U = L g L^T (first step of Sec. 4.3) for w [K][C][3][3] into that caller-owned, 256-byte
 * aligned device buffer, laid out [(m+2)^2][C rounded up to 16][K rounded up to 32] with zeros
 * in the padding.  conv_winograd_pre: conv_winograd_ws with U in place of w; the workspace
 * size is the one conv_winograd_workspace_bytes reports. */
size_t conv_winograd_kernel_bytes(int C, int K, int m);
int conv_winograd_transform_kernels(const float* w, float* U, int C, int K, int m);
int conv_winograd_pre(const float* x, const float* U, float* y,
                      int N, int C, int H, int W, int K, int m,
                      void* workspace, size_t workspace_bytes, const iolb_tile_config* cfg);

/* The analytical tuner.  Searching domain: Table 1 of Sec. 6.2 read for this machine (tile extents from the
 * factors of the output extents, blocks that fit the accumulator registers and the LDS).  Order: a modelled
 * run time -- THIS LIBRARY'S HEURISTIC, fitted to tile sweeps on an MI355X -- whose memory term and tie-break
 * are the reading volume of the dataflow of Sec. 5.2 / 5.3.  Host only; shape and out are host pointers.
 * lds_bytes: LDS available to one workgroup; 0 = automatic: 81920 (half a compute unit's LDS, the
 * "two blocks per multiprocessor" rule of Sec. 6.2), or the whole LDS for tiles whose registers
 * allow only one workgroup per compute unit anyway.  vgpr_budget: accumulator registers per
 * lane (0 = default 128; the fused Winograd blocks, which hold up to 96, are exempt from the default).
 * IOLB_ENOTILE when nothing fits. */
int iolb_tune(const iolb_shape* shape, size_t lds_bytes, int vgpr_budget, iolb_tile_config* out);

/* The bound-only pick: the same domain restricted to the optimality box of Table 1 (z <= sqrt(S_b/rho),
 * x y <= sqrt(S_b rho); the whole domain if the box is empty), ordered by the paper's objective alone -- the
 * reading volume Q_read of Sec. 5.2 / 5.3 evaluated exactly for the tile, ties by |b x y mu^2 - W_ker H_ker z|
 * (distance from the optimality condition x y = R z), then the fuller block.  For the Winograd algos the fused
 * dataflow of Sec. 5.3 comes before the unfused tiles.  Same arguments and errors as iolb_tune. */
int iolb_tune_bound(const iolb_shape* shape, size_t lds_bytes, int vgpr_budget, iolb_tile_config* out);

/* Every feasible tile for the shape, best first (the domain the exhaustive sweep times).
 * use_box != 0 applies the optimality-condition box z <= sqrt(S_b/rho), xy <= sqrt(S_b rho).
 * Writes at most `capacity` entries to out (may be NULL) and returns the total count, or a
 * negative code. */
int64_t iolb_enumerate(const iolb_shape* shape, size_t lds_bytes, int vgpr_budget, int use_box,
                       iolb_tile_config* out, int64_t capacity);

/* Lower-bound figures for a layer at fast-memory size S_f elements.  Host only. */
int iolb_bounds(const iolb_shape* shape, int64_t S_f_elems, iolb_bounds_out* out);

/* The constant transform matrices the Winograd kernels use for F(m x m, 3 x 3) (Sec. 2.3: input
 * transform B d B^T, kernel transform L g L^T, output transform A M A^T), row-major into host
 * arrays A[m][m+2], L[m+2][3], B[m+2][m+2].  Host only.  IOLB_EUNSUPPORTED for other m. */
int iolb_winograd_matrices(int m, float* A, float* L, float* B);

/* Stream (a hipStream_t) later calls enqueue on; NULL selects the null stream. */
int iolb_set_stream(void* hip_stream);

/* Timing hook for benchmarks: when enabled, the main kernel of each conv call is bracketed by
 * HIP events on the call's stream.  Kinds: the direct-convolution kernel (IOLB_TIME_DIRECT), the
 * Winograd batched product (IOLB_TIME_WINO_PRODUCT) and the fused Winograd matrix-core kernel
 * (IOLB_TIME_WINO_FUSED).  iolb_timing_read waits for the recorded
 * events of one kind, returns how many launches were timed since the last read of that kind and
 * their total duration in milliseconds, and forgets them. */
enum { IOLB_TIME_DIRECT = 0, IOLB_TIME_WINO_PRODUCT = 1, IOLB_TIME_WINO_FUSED = 2 };
int iolb_timing_enable(int on);
int iolb_timing_read(int kind, int* launches, float* total_ms);

/* Ceiling probes for roofline reports (the experimental set-up of Sec. 7 quotes peak rates; these measure
 * what the device at hand delivers).  Both run `reps` launches on the set stream after one untimed launch,
 * wait for them, and return the average duration of a launch in milliseconds.
 *   iolb_probe_hbm_copy: a streaming copy of `bytes` (a multiple of 16) from src to dst, device buffers
 *     that do not overlap; the traffic of a launch is 2 * bytes.
 *   iolb_probe_mfma_f32: a loop of independent v_mfma_f32_32x32x2_f32 with operands in registers; `sink`
 *     is a device buffer of at least iolb_probe_mfma_sink_bytes() bytes that receives the accumulators'
 *     sums; *flop_per_launch gets the floating-point operations of one launch.
 * IOLB_EINVAL for null pointers, bytes == 0 or not a multiple of 16, iters < 1, reps < 1. */
int iolb_probe_hbm_copy(const void* src, void* dst, size_t bytes, int reps, float* ms_per_launch);
size_t iolb_probe_mfma_sink_bytes(void);
int iolb_probe_mfma_f32(void* sink, int iters, int reps, float* ms_per_launch, double* flop_per_launch);

/* Probe of how the waves of one SIMD share its fp32 pipeline (the fused Winograd kernels of Sec. 5.3 mix matrix
 * and plain vector arithmetic in one workgroup; this measures what that costs).  One launch of 256 workgroups of
 * 4 * slots waves, so that every SIMD holds `slots` waves (1..4); the waves of slot s run roles[s] (a host array):
 * IOLB_PROBE_ROLE_MFMA = `iters` rounds of 8 v_mfma_f32_32x32x2_f32 (512 matrix cycles per round),
 * IOLB_PROBE_ROLE_VALU = `iters` rounds of 64 v_fma_f32.  `scratch` is a device buffer of at least
 * iolb_probe_share_scratch_bytes() bytes.  *ms gets the duration of the launch, ticks_per_slot[s] (host, `slots`
 * doubles) the average clock ticks a wave of slot s spent in its loop.  Runs on the set stream and waits for it.
 * IOLB_EINVAL for null pointers, slots outside 1..4, an unknown role, iters < 1. */
enum { IOLB_PROBE_ROLE_MFMA = 0, IOLB_PROBE_ROLE_VALU = 1 };
size_t iolb_probe_share_scratch_bytes(void);
int iolb_probe_pipeline_share(void* scratch, int slots, const int* roles, int iters, float* ms, double* ticks_per_slot);

/* Waits for the current GPU and frees the library's workspaces on it (all streams, and the buffers larger ones
 * have replaced); they are otherwise kept until the process ends.  Graphs captured from calls that used them
 * must not be replayed afterwards. */
int iolb_release_workspace(void);

const char* iolb_strerror(int code);
/* Text of the last HIP error seen by this thread's calls ("" if none). */
const char* iolb_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* IOLBCONV_H */
