// C-ABI layer: argument checks, tile selection, workspace, launches.  See include/iolbconv.h.
#include <hip/hip_runtime.h>

#include <array>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <tuple>
#include <vector>

#include "iolbconv.h"
#include "kernels.h"
#include "tune.h"
#include "wino_mats.h"

namespace {

thread_local hipStream_t t_stream = nullptr;
thread_local std::string t_hip_error;

int hip_fail(hipError_t e)
{
    t_hip_error = hipGetErrorString(e);
    return IOLB_EHIP;
}
#define IOLB_HIP(call)                                \
    do {                                              \
        hipError_t e__ = (call);                      \
        if (e__ != hipSuccess) return hip_fail(e__);  \
    } while (0)

struct Workspace {
    void* ptr = nullptr;
    size_t bytes = 0;
};
struct DeviceState {
    std::map<hipStream_t, Workspace> ws;   // the library's workspace: one per stream that has called in
    std::vector<void*> retired;            // buffers a larger one has replaced: kept until iolb_release_workspace,
                                           // because launches in flight and captured graphs may still name them
    float* scratch = nullptr;              // this device's copy of the static scratch array (conv_direct_noalloc)
};

// Scratch of the entry point that allocates nothing: the re-laid-out weights of one layer.  Every GPU the
// library runs on holds its own copy of the array, at its own address, until the process ends.
constexpr size_t kScratchFloats = (size_t)4 << 20;            // 16 MiB
static __device__ __align__(256) float scratch[kScratchFloats];
std::mutex g_mutex;
std::map<int, DeviceState> g_devices;

int device_state(DeviceState** out)
{
    int dev = 0;
    IOLB_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_mutex);
    *out = &g_devices[dev];
    return IOLB_OK;
}

// Library-owned workspace of the calling thread's stream on the current device: grown on demand, never freed
// before iolb_release_workspace.  One workspace per stream makes calls on different streams independent (one
// stream per host thread); two calls on ONE stream are ordered by the stream.  A buffer that has to grow is
// replaced, not freed: kernels already enqueued, and graphs captured earlier, keep a valid address.
int ensure_workspace(DeviceState* d, size_t bytes, void** out)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    Workspace& w = d->ws[t_stream];
    if (w.bytes < bytes) {
        void* p = nullptr;
        IOLB_HIP(hipMalloc(&p, bytes));
        if (w.ptr) d->retired.push_back(w.ptr);
        w.ptr = p;
        w.bytes = bytes;
    }
    *out = w.ptr;
    return IOLB_OK;
}

// Device address of this device's scratch array, looked up once per device (with that device current: the caller
// has just asked for it with hipGetDevice).  In host code the array's name is only a handle for this lookup.
int scratch_address(DeviceState* d, float** out)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    if (!d->scratch) {
        void* p = nullptr;
        IOLB_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        d->scratch = static_cast<float*>(p);
    }
    *out = d->scratch;
    return IOLB_OK;
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// ---- timing hook --------------------------------------------------------------------------
bool g_timing = false;
std::vector<std::pair<hipEvent_t, hipEvent_t>> g_events[3];

struct MainKernelTimer {
    hipEvent_t a = nullptr, b = nullptr;
    bool on;
    int kind;
    MainKernelTimer(hipStream_t st, int kind_) : on(g_timing), kind(kind_)
    {
        if (!on) return;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { on = false; return; }
        hipEventRecord(a, st);
    }
    void stop(hipStream_t st)
    {
        if (!on) return;
        hipEventRecord(b, st);
        { std::lock_guard<std::mutex> lock(g_mutex); g_events[kind].emplace_back(a, b); }
    }
};

// ---- tile cache -----------------------------------------------------------------------------
typedef std::tuple<int, int, int, int, int, int, int, int, int, int> ShapeKey;
std::map<ShapeKey, iolb_tile_config> g_tiles;

// Tiles of the kernels that exist for one kind of call only: IOLB_PATH_POINT (channels-outermost tensors, no
// padding on either axis) and the thin direct layers (wt_mode 2: channels-outermost tensors).
bool is_thin(const iolb_tile_config& c) { return c.path == IOLB_PATH_FMA && c.wt_mode == 2; }

// pointwise_ok / thin_ok = false: the call cannot run such a tile: the best of the others.
int tuned_tile(const iolb_shape& s, iolb_tile_config* cfg, bool pointwise_ok = true, bool thin_ok = true)
{
    const ShapeKey key(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.algo + (pointwise_ok ? 0 : 1000) + (thin_ok ? 0 : 2000));
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        auto it = g_tiles.find(key);
        if (it != g_tiles.end()) { *cfg = it->second; return IOLB_OK; }
    }
    int rc = iolb::tune(s, 0, 0, cfg);
    if (rc != IOLB_OK) return rc;
    if ((!pointwise_ok && cfg->path == IOLB_PATH_POINT) || (!thin_ok && is_thin(*cfg))) {
        std::vector<iolb::Candidate> all;
        rc = iolb::enumerate(s, 0, 0, false, &all);
        if (rc != IOLB_OK) return rc;
        const iolb::Candidate* first = nullptr;
        for (const auto& c : all)
            if ((pointwise_ok || c.cfg.path != IOLB_PATH_POINT) && (thin_ok || !is_thin(c.cfg))) { first = &c; break; }
        if (!first) return IOLB_ENOTILE;
        *cfg = first->cfg;
    }
    std::lock_guard<std::mutex> lock(g_mutex);
    g_tiles[key] = *cfg;
    return IOLB_OK;
}

bool same_config(const iolb_tile_config& a, const iolb_tile_config& b)
{
    return a.b == b.b && a.x == b.x && a.y == b.y && a.z == b.z && a.alpha == b.alpha && a.threads == b.threads &&
           a.waves_m == b.waves_m && a.waves_n == b.waves_n && a.path == b.path && a.wt_mode == b.wt_mode &&
           a.lds_bytes_used == b.lds_bytes_used && a.acc_regs_per_thread == b.acc_regs_per_thread &&
           a.q_read_elems == b.q_read_elems && a.q_write_elems == b.q_write_elems;
}

// A caller-supplied tile must be one the enumeration produces for this shape (any LDS budget up to the
// whole compute unit), so that every kernel assumption about it holds.  Accepted (shape, tile) pairs are
// remembered: sweeps call the same tile many times.
typedef std::tuple<ShapeKey, std::array<int64_t, 14>> CheckedKey;
std::map<CheckedKey, bool> g_checked;

int check_config(const iolb_shape& s, const iolb_tile_config& cfg)
{
    const CheckedKey key(ShapeKey(s.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad, s.algo),
                         std::array<int64_t, 14>{cfg.b, cfg.x, cfg.y, cfg.z, cfg.alpha, cfg.threads, cfg.waves_m,
                                                 cfg.waves_n, cfg.path, cfg.wt_mode, cfg.lds_bytes_used,
                                                 cfg.acc_regs_per_thread, cfg.q_read_elems, cfg.q_write_elems});
    {
        std::lock_guard<std::mutex> lock(g_mutex);
        if (g_checked.count(key)) return IOLB_OK;
    }
    std::vector<iolb::Candidate> all;
    const int rc = cfg.path == IOLB_PATH_FMA && s.algo == IOLB_DIRECT && cfg.wt_mode != 2 ? iolb::enumerate_fma(s, 160 * 1024, 0, &all)
                                                                      : iolb::enumerate(s, 160 * 1024, 0, false, &all);
    if (rc != IOLB_OK) return rc;
    for (const auto& c : all) {
        iolb_tile_config probe = c.cfg;
        // alpha may be any shallower stage depth than the enumeration's (a multiple of 4 on the MFMA path)
        // (the stage depths of the 1 x 1 kernel are enumerated one by one)
        if (cfg.path != IOLB_PATH_POINT && cfg.alpha >= 1 && cfg.alpha <= c.cfg.alpha &&
            (cfg.path == IOLB_PATH_FMA || cfg.alpha % 4 == 0) && c.cfg.alpha % cfg.alpha == 0) {
            probe.alpha = cfg.alpha;
            // a single-stage tile counts one buffer, a shallower (multi-stage) depth two
            const int64_t buffers = cfg.path == IOLB_PATH_MFMA && c.cfg.alpha >= s.C && cfg.alpha < s.C ? 2 : 1;
            probe.lds_bytes_used = (int32_t)((int64_t)c.cfg.lds_bytes_used / c.cfg.alpha * cfg.alpha * buffers);
        }
        if (same_config(probe, cfg)) {
            std::lock_guard<std::mutex> lock(g_mutex);
            g_checked[key] = true;
            return IOLB_OK;
        }
    }
    return IOLB_EINVAL;
}

// layout CWH: s, P, Q describe the transposed layer (H and W, R and S exchanged) and the weights are read
// transposed; the tensors are then plain CHW tensors of that layer.
// wt_buf != nullptr: room for the re-laid-out weights (wt_floats floats) given by the caller, so that nothing is
// allocated; otherwise the library's workspace is used.
int run_direct(const float* x, const float* w, float* y, const iolb_shape& s, int P, int Q, const iolb_tile_config& cfg,
               int layout = IOLB_LAYOUT_CHW, int pad_w = -1, float* wt_buf = nullptr, size_t wt_floats = 0)
{
    DeviceState* dev = nullptr;
    int rc = device_state(&dev);
    if (rc != IOLB_OK) return rc;
    if (cfg.path == IOLB_PATH_POINT) {
        // 1 x 1, no padding, channels outermost: the output plane as one row of P * Q pixels
        if (layout != IOLB_LAYOUT_CHW || (pad_w >= 0 && pad_w != 0) || s.pad != 0 || s.R != 1 || s.S != 1)
            return IOLB_EINVAL;
        iolb::PointGeom g{};
        g.N = s.N; g.C = s.C; g.HW = P * Q; g.K = s.K;
        g.HWin = s.H * s.W; g.Win = s.W; g.Q = Q; g.stride = s.stride;
        g.z = cfg.z; g.mbw = cfg.z / 32; g.nbw = cfg.x / 128; g.waves = 4; g.alpha = cfg.alpha;
        if (cfg.threads != 256 || cfg.z != 32 * g.mbw || cfg.x != 128 * g.nbw || cfg.alpha < 1) return IOLB_EINVAL;
        g.Kp = (s.K + cfg.z - 1) / cfg.z * cfg.z;
        g.nbk = g.Kp / cfg.z;
        g.tiles_per_image = (g.HW + 32 * g.nbw - 1) / (32 * g.nbw);
        const int64_t ntiles = (int64_t)s.N * g.tiles_per_image;
        if ((ntiles + 3) / 4 * g.nbk > 0x7fffffffLL) return IOLB_EINVAL;
        g.npg = (int)((ntiles + 3) / 4);
        // the kernel reads w itself when its rows are whole 16-byte pieces; otherwise a copy padded with zeros
        g.Cw = (s.C + 3) / 4 * 4;
        hipStream_t st = t_stream;
        const float* wk = w;
        if (g.Cw != s.C || (reinterpret_cast<size_t>(w) & 15)) {
            const size_t wbytes = sizeof(float) * (size_t)s.K * g.Cw;
            float* wp = wt_buf;
            if (wt_buf) {
                if (wbytes > sizeof(float) * wt_floats) return IOLB_EWORKSPACE;
            } else {
                void* ws = nullptr;
                rc = ensure_workspace(dev, align256(wbytes), &ws);
                if (rc != IOLB_OK) return rc;
                wp = static_cast<float*>(ws);
            }
            IOLB_HIP(iolb::launch_pointwise_weight_pad(w, wp, s.K, s.C, g.Cw, st));
            wk = wp;
        }
        MainKernelTimer timer(st, IOLB_TIME_DIRECT);
        IOLB_HIP(iolb::launch_pointwise_mfma(x, wk, y, g, st));
        timer.stop(st);
        return IOLB_OK;
    }
    iolb::DirectGeom g{};
    g.N = s.N; g.C = s.C; g.H = s.H; g.W = s.W; g.K = s.K; g.R = s.R; g.S = s.S; g.stride = s.stride; g.pad = s.pad;
    g.pad_w = pad_w < 0 ? s.pad : pad_w;
    g.P = P; g.Q = Q;
    if (is_thin(cfg)) {
        // 3 x 3, stride 1, C <= 4, channels outermost: one lane per few pixels and all output channels
        if (layout != IOLB_LAYOUT_CHW || s.R != 3 || s.S != 3 || s.stride != 1 || s.C > 4 || cfg.z != s.K || cfg.alpha != s.C)
            return IOLB_EINVAL;
        const size_t wbytes = sizeof(float) * (size_t)s.K * iolb::direct_thin_row(s.C);
        float* wk = wt_buf;
        if (wt_buf) {
            if (wbytes > sizeof(float) * wt_floats) return IOLB_EWORKSPACE;
        } else {
            void* ws = nullptr;
            rc = ensure_workspace(dev, align256(wbytes), &ws);
            if (rc != IOLB_OK) return rc;
            wk = static_cast<float*>(ws);
        }
        hipStream_t st = t_stream;
        IOLB_HIP(iolb::launch_direct_thin_rows(w, wk, s.K, s.C, st));
        IOLB_HIP(iolb::launch_direct_thin(x, wk, y, g, st));       // a plain-FMA kernel: not timed with the matrix-core ones
        return IOLB_OK;
    }
    g.b = cfg.b; g.tx = cfg.x; g.ty = cfg.y; g.z = cfg.z; g.alpha = cfg.alpha;
    g.threads = cfg.threads; g.waves_m = cfg.waves_m; g.waves_n = cfg.waves_n;
    g.per_thread = cfg.acc_regs_per_thread;
    g.Kp = cfg.path == IOLB_PATH_MFMA ? (s.K + 31) / 32 * 32 : s.K;
    g.nbx = (Q + cfg.x - 1) / cfg.x; g.nby = (P + cfg.y - 1) / cfg.y; g.nbn = s.N / cfg.b; g.nbk = g.Kp / cfg.z;   // edge tiles may hang over
    g.xh = (cfg.x - 1) * s.stride + s.S;
    g.yh = (cfg.y - 1) * s.stride + s.R;
    g.halo = cfg.b * g.xh * g.yh;
    g.hwc = layout == IOLB_LAYOUT_HWC;
    g.w_transposed = layout == IOLB_LAYOUT_CWH;
    if ((int64_t)g.nbx * g.nby * g.nbn * g.nbk > 0x7fffffffLL) return IOLB_EINVAL;
    hipStream_t st = t_stream;
    if (cfg.path == IOLB_PATH_MFMA) {
        const int c_padded = (s.C + cfg.alpha - 1) / cfg.alpha * cfg.alpha;     // whole stages
        const size_t wbytes = sizeof(float) * (size_t)g.Kp * c_padded * s.R * s.S;
        float* wt = wt_buf;
        if (wt_buf) {
            if (wbytes > sizeof(float) * wt_floats) return IOLB_EWORKSPACE;
        } else {
            void* ws = nullptr;
            rc = ensure_workspace(dev, align256(wbytes), &ws);
            if (rc != IOLB_OK) return rc;
            wt = static_cast<float*>(ws);
        }
        if (g.w_transposed)
            IOLB_HIP(iolb::launch_weight_relayout_transposed(w, wt, s.K, g.Kp, s.C, s.R, s.S, c_padded * s.R * s.S, st));
        else
            IOLB_HIP(iolb::launch_weight_relayout(w, wt, s.K, g.Kp, s.C * s.R * s.S, c_padded * s.R * s.S, st));
        MainKernelTimer timer(st, IOLB_TIME_DIRECT);
        IOLB_HIP(g.hwc ? iolb::launch_direct_mfma_hwc(x, wt, y, g, st) : iolb::launch_direct_mfma(x, wt, y, g, st));
        timer.stop(st);
    } else {
        MainKernelTimer timer(st, IOLB_TIME_DIRECT);
        IOLB_HIP(iolb::launch_direct_fma(x, w, y, g, st));
        timer.stop(st);
    }
    return IOLB_OK;
}

int winograd_geom(const iolb_shape& s, const iolb_tile_config& cfg, iolb::WinoGeom* g)
{
    const int m = iolb::winograd_m(s.algo);
    g->N = s.N; g->C = s.C; g->H = s.H; g->W = s.W; g->K = s.K; g->m = m;
    g->pad = s.pad;
    g->P = s.H + 2 * s.pad - 2;
    g->Q = s.W + 2 * s.pad - 2;
    g->th = (g->P + m - 1) / m;
    g->tw = (g->Q + m - 1) / m;
    const int64_t tiles = (int64_t)s.N * g->th * g->tw;
    g->tb = cfg.x / m;
    g->z = cfg.z;
    g->alpha = cfg.alpha;
    g->Cp = (s.C + cfg.alpha - 1) / cfg.alpha * cfg.alpha;
    // the fused matrix-core kernel covers K with whole z-channel blocks, the other paths with 32-channel blocks
    g->Kp = cfg.path == IOLB_PATH_FUSED ? (s.K + cfg.z - 1) / cfg.z * cfg.z : (s.K + 31) / 32 * 32;
    g->CpU = g->Cp;
    g->waves_m = cfg.waves_m;
    g->waves_n = cfg.waves_n;
    const int64_t pitch = (tiles + g->tb - 1) / g->tb * g->tb;
    const int64_t n2 = (int64_t)(m + 2) * (m + 2);
    // V and M of the unfused path are indexed with 32-bit element counts
    if (cfg.path == IOLB_PATH_MFMA && (n2 * g->Cp * pitch >= (1LL << 31) || n2 * g->Kp * pitch >= (1LL << 31))) return IOLB_EINVAL;
    if (n2 * g->Cp * g->Kp >= (1LL << 31)) return IOLB_EINVAL;
    g->tiles = (int)tiles;
    g->tiles_pitch = (int)pitch;
    return IOLB_OK;
}

struct WinoWorkspace {
    size_t u_off, v_off, m_off, total;
};
// path: the tile's path.  IOLB_PATH_MFMA (unfused): U, V, M.  IOLB_PATH_FMA (thin layers, one kernel with the
// transformed inputs and the channel sums in registers): U and, in V's place, U again as one row per output
// channel.  IOLB_PATH_FUSED (one matrix-core kernel): U in the channel-pair layout and, in V's place, room
// for a second copy (used when the caller brings plane-major transformed kernels).
WinoWorkspace winograd_layout(int C, int K, int m, int64_t tiles_pitch, int path = IOLB_PATH_MFMA)
{
    const size_t n2 = (size_t)(m + 2) * (m + 2);
    const size_t ubytes = align256(sizeof(float) * n2 * C * K);
    WinoWorkspace l;
    l.u_off = 0;
    l.v_off = l.u_off + ubytes;
    if (path == IOLB_PATH_FMA) {
        l.m_off = l.v_off + align256(sizeof(float) * K * iolb::wino_fused_row(m, C));
        l.total = l.m_off;
    } else if (path == IOLB_PATH_FUSED) {
        l.m_off = l.v_off + ubytes;
        l.total = l.m_off;
    } else {
        l.m_off = l.v_off + align256(sizeof(float) * n2 * C * tiles_pitch);
        l.total = l.m_off + align256(sizeof(float) * n2 * K * tiles_pitch);
    }
    return l;
}

// Largest workspace any tile of the enumeration can ask for: unfused blocks hold at most 1024 sub-domains and
// stages at most 16 channels; the fused matrix-core blocks cover K with blocks of up to 64 channels.
size_t winograd_workspace_max(int C, int K, int m, int64_t tiles)
{
    const size_t unfused = winograd_layout(C + 15, (K + 31) / 32 * 32, m, tiles + 1024).total;
    const size_t fused = winograd_layout(C + 15, (K + 63) / 64 * 64, m, 0, IOLB_PATH_FUSED).total;
    return unfused > fused ? unfused : fused;
}

int make_wino_shape(int N, int C, int H, int W, int K, int m, iolb_shape* s, int pad = 1)
{
    int algo = 0;
    switch (m) {
    case 2: algo = IOLB_WINO_F2; break;
    case 3: algo = IOLB_WINO_F3; break;
    case 4: algo = IOLB_WINO_F4; break;
    case 6: algo = IOLB_WINO_F6; break;
    default: return IOLB_EUNSUPPORTED;
    }
    *s = iolb_shape{N, C, H, W, K, 3, 3, 1, pad, algo};
    int P = 0, Q = 0;
    return iolb::validate_shape(*s, &P, &Q);
}

// Channel rows per plane of a caller-held transformed-kernel buffer: every stage depth divides 16.
int pretransformed_rows(int C) { return (C + 15) / 16 * 16; }

// w != nullptr: transform the kernels into the workspace first.  w == nullptr: Upre holds them already
// (written by conv_winograd_transform_kernels).
int run_winograd(const float* x, const float* w, const float* Upre, float* y, const iolb_shape& s,
                 const iolb_tile_config& cfg, void* ws, size_t ws_bytes)
{
    DeviceState* dev = nullptr;
    int rc = device_state(&dev);
    if (rc != IOLB_OK) return rc;
    iolb::WinoGeom g{};
    rc = winograd_geom(s, cfg, &g);
    if (rc != IOLB_OK) return rc;
    const bool fused = cfg.path == IOLB_PATH_FMA;
    const WinoWorkspace l = winograd_layout(g.Cp, g.Kp, g.m, g.tiles_pitch, cfg.path);
    if (!ws || ws_bytes < l.total || (reinterpret_cast<uintptr_t>(ws) & 255)) return IOLB_EWORKSPACE;
    char* base = static_cast<char*>(ws);
    float* U = reinterpret_cast<float*>(base + l.u_off);
    float* V = reinterpret_cast<float*>(base + l.v_off);
    float* M = reinterpret_cast<float*>(base + l.m_off);
    hipStream_t st = t_stream;
    const float* Uuse = U;
    if (cfg.path == IOLB_PATH_FUSED) {
        // the transformed kernels in the channel-pair layout: made from w, or re-laid out from the caller's
        if (w) {
            IOLB_HIP(iolb::launch_wino_kernel_transform_paired(w, U, g, st));
        } else {
            IOLB_HIP(iolb::launch_wino_pair_relayout(Upre, pretransformed_rows(s.C), (s.K + 31) / 32 * 32, V, g, st));
            Uuse = V;
        }
        MainKernelTimer timer(st, IOLB_TIME_WINO_FUSED);
        IOLB_HIP(iolb::launch_wino_fused_mfma(x, Uuse, y, g, st));
        timer.stop(st);
        return IOLB_OK;
    }
    if (w) {
        IOLB_HIP(iolb::launch_wino_kernel_transform(w, U, g, st));
    } else {
        g.CpU = pretransformed_rows(s.C);
        Uuse = Upre;
    }
    if (fused) {
        IOLB_HIP(iolb::launch_wino_fused_relayout(Uuse, V, g, st));
        IOLB_HIP(iolb::launch_wino_fused(x, V, y, g, st));
        return IOLB_OK;
    }
    IOLB_HIP(iolb::launch_wino_input_transform(x, V, g, st));
    MainKernelTimer timer(st, IOLB_TIME_WINO_PRODUCT);
    IOLB_HIP(iolb::launch_wino_product(Uuse, V, M, g, st));
    timer.stop(st);
    IOLB_HIP(iolb::launch_wino_output_transform(M, y, g, st));
    return IOLB_OK;
}

// Runs `launch` once untimed and then `reps` times between two events on the set stream.
template <typename Launch>
int time_probe(int reps, float* ms_per_launch, Launch launch)
{
    hipEvent_t e0 = nullptr, e1 = nullptr;
    IOLB_HIP(launch());                                   // untimed: clocks up, code loaded
    IOLB_HIP(hipEventCreate(&e0));
    hipError_t e = hipEventCreate(&e1);
    if (e == hipSuccess) e = hipEventRecord(e0, t_stream);
    for (int r = 0; r < reps && e == hipSuccess; ++r) e = launch();
    if (e == hipSuccess) e = hipEventRecord(e1, t_stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (e != hipSuccess) return hip_fail(e);
    *ms_per_launch = ms / reps;
    return IOLB_OK;
}

}  // namespace

extern "C" {

int conv_direct_cfg(const float* x, const float* w, float* y, int N, int C, int H, int W, int K, int R, int S,
                    int stride, int pad, const iolb_tile_config* cfg)
{
    if (!x || !w || !y || !cfg) return IOLB_EINVAL;
    const iolb_shape s{N, C, H, W, K, R, S, stride, pad, IOLB_DIRECT};
    int P = 0, Q = 0;
    int rc = iolb::validate_shape(s, &P, &Q);
    if (rc != IOLB_OK) return rc;
    rc = check_config(s, *cfg);
    if (rc != IOLB_OK) return rc;
    return run_direct(x, w, y, s, P, Q, *cfg);
}

int conv_direct(const float* x, const float* w, float* y, int N, int C, int H, int W, int K, int R, int S,
                int stride, int pad)
{
    if (!x || !w || !y) return IOLB_EINVAL;
    const iolb_shape s{N, C, H, W, K, R, S, stride, pad, IOLB_DIRECT};
    int P = 0, Q = 0;
    int rc = iolb::validate_shape(s, &P, &Q);
    if (rc != IOLB_OK) return rc;
    iolb_tile_config cfg;
    rc = tuned_tile(s, &cfg);
    if (rc != IOLB_OK) return rc;
    return run_direct(x, w, y, s, P, Q, cfg);
}

int conv_direct_noalloc(const float* x, const float* w, float* y, int N, int C, int H, int W, int K, int R, int S,
                        int stride, int pad)
{
    if (!x || !w || !y) return IOLB_EINVAL;
    const iolb_shape s{N, C, H, W, K, R, S, stride, pad, IOLB_DIRECT};
    int P = 0, Q = 0;
    int rc = iolb::validate_shape(s, &P, &Q);
    if (rc != IOLB_OK) return rc;
    iolb_tile_config cfg;
    rc = tuned_tile(s, &cfg);
    if (rc != IOLB_OK) return rc;
    DeviceState* dev = nullptr;
    rc = device_state(&dev);
    if (rc != IOLB_OK) return rc;
    float* buf = nullptr;
    rc = scratch_address(dev, &buf);
    if (rc != IOLB_OK) return rc;
    // the limit is checked inside run_direct, before anything is launched: IOLB_EWORKSPACE beyond it
    return run_direct(x, w, y, s, P, Q, cfg, IOLB_LAYOUT_CHW, -1, buf, kScratchFloats);
}

size_t conv_direct_noalloc_max_weight_floats(void) { return kScratchFloats; }

int conv_direct_pad2(const float* x, const float* w, float* y, int N, int C, int H, int W, int K, int R, int S,
                     int stride, int pad_h, int pad_w)
{
    if (!x || !w || !y) return IOLB_EINVAL;
    if (pad_h < 0 || pad_w < 0) return IOLB_EINVAL;
    // The tile depends on the layer through its output extents only: tune the layer whose image already
    // contains the zero borders (H + 2 pad_h by W + 2 pad_w, no padding), run the real one.
    if ((int64_t)H + 2LL * pad_h > 0x7fffffffLL || (int64_t)W + 2LL * pad_w > 0x7fffffffLL) return IOLB_EINVAL;
    const iolb_shape bordered{N, C, H + 2 * pad_h, W + 2 * pad_w, K, R, S, stride, 0, IOLB_DIRECT};
    int P = 0, Q = 0;
    int rc = iolb::validate_shape(bordered, &P, &Q);
    if (rc != IOLB_OK) return rc;
    if (H < 1 || W < 1) return IOLB_EINVAL;
    iolb_tile_config cfg;
    rc = tuned_tile(bordered, &cfg, pad_h == 0 && pad_w == 0);
    if (rc != IOLB_OK) return rc;
    const iolb_shape s{N, C, H, W, K, R, S, stride, pad_h, IOLB_DIRECT};
    return run_direct(x, w, y, s, P, Q, cfg, IOLB_LAYOUT_CHW, pad_w);
}

int conv_direct_layout(const float* x, const float* w, float* y, int N, int C, int H, int W, int K, int R, int S,
                       int stride, int pad, int layout, const iolb_tile_config* cfg)
{
    if (!x || !w || !y) return IOLB_EINVAL;
    if (layout != IOLB_LAYOUT_CHW && layout != IOLB_LAYOUT_HWC && layout != IOLB_LAYOUT_CWH) return IOLB_EUNSUPPORTED;
    // CWH: the W x H image convolved with the transposed kernels, as a CHW layer
    const bool cwh = layout == IOLB_LAYOUT_CWH;
    const iolb_shape s{N, C, cwh ? W : H, cwh ? H : W, K, cwh ? S : R, cwh ? R : S, stride, pad, IOLB_DIRECT};
    int P = 0, Q = 0;
    int rc = iolb::validate_shape(s, &P, &Q);
    if (rc != IOLB_OK) return rc;
    iolb_tile_config tile;
    if (cfg) {
        rc = check_config(s, *cfg);
        if (rc != IOLB_OK) return rc;
        tile = *cfg;
    } else {
        rc = tuned_tile(s, &tile, layout == IOLB_LAYOUT_CHW, layout == IOLB_LAYOUT_CHW);
        if (rc != IOLB_OK) return rc;
    }
    return run_direct(x, w, y, s, P, Q, tile, layout);
}

size_t conv_winograd_workspace_bytes(int N, int C, int H, int W, int K, int m)
{
    iolb_shape s;
    if (make_wino_shape(N, C, H, W, K, m, &s) != IOLB_OK) return 0;
    // large enough for every tile the enumeration can produce
    const int64_t tiles = (int64_t)N * ((H + m - 1) / m) * ((W + m - 1) / m);
    return winograd_workspace_max(C, K, m, tiles);
}

int conv_winograd_ws(const float* x, const float* w, float* y, int N, int C, int H, int W, int K, int m,
                     void* workspace, size_t workspace_bytes, const iolb_tile_config* cfg)
{
    if (!x || !w || !y) return IOLB_EINVAL;
    iolb_shape s;
    int rc = make_wino_shape(N, C, H, W, K, m, &s);
    if (rc != IOLB_OK) return rc;
    iolb_tile_config tile;
    if (cfg) {
        rc = check_config(s, *cfg);
        if (rc != IOLB_OK) return rc;
        tile = *cfg;
    } else {
        rc = tuned_tile(s, &tile);
        if (rc != IOLB_OK) return rc;
    }
    return run_winograd(x, w, nullptr, y, s, tile, workspace, workspace_bytes);
}

size_t conv_winograd_kernel_bytes(int C, int K, int m)
{
    if (C < 1 || K < 1 || (m != 2 && m != 3 && m != 4 && m != 6)) return 0;
    return sizeof(float) * (size_t)(m + 2) * (m + 2) * pretransformed_rows(C) * ((K + 31) / 32 * 32);
}

int conv_winograd_transform_kernels(const float* w, float* U, int C, int K, int m)
{
    if (!w || !U || C < 1 || K < 1) return IOLB_EINVAL;
    if (m != 2 && m != 3 && m != 4 && m != 6) return IOLB_EUNSUPPORTED;
    if ((int64_t)K * C * 9 >= (1LL << 31) || conv_winograd_kernel_bytes(C, K, m) / sizeof(float) >= ((size_t)1 << 31))
        return IOLB_EINVAL;
    iolb::WinoGeom g{};
    g.C = C; g.K = K; g.m = m;
    g.Kp = (K + 31) / 32 * 32;
    g.CpU = pretransformed_rows(C);
    IOLB_HIP(iolb::launch_wino_kernel_transform(w, U, g, t_stream));
    return IOLB_OK;
}

int conv_winograd_pre(const float* x, const float* U, float* y, int N, int C, int H, int W, int K, int m,
                      void* workspace, size_t workspace_bytes, const iolb_tile_config* cfg)
{
    if (!x || !U || !y) return IOLB_EINVAL;
    iolb_shape s;
    int rc = make_wino_shape(N, C, H, W, K, m, &s);
    if (rc != IOLB_OK) return rc;
    iolb_tile_config tile;
    if (cfg) {
        rc = check_config(s, *cfg);
        if (rc != IOLB_OK) return rc;
        tile = *cfg;
    } else {
        rc = tuned_tile(s, &tile);
        if (rc != IOLB_OK) return rc;
    }
    return run_winograd(x, nullptr, U, y, s, tile, workspace, workspace_bytes);
}

int conv_winograd(const float* x, const float* w, float* y, int N, int C, int H, int W, int K, int m)
{
    if (!x || !w || !y) return IOLB_EINVAL;
    iolb_shape s;
    int rc = make_wino_shape(N, C, H, W, K, m, &s);
    if (rc != IOLB_OK) return rc;
    iolb_tile_config tile;
    rc = tuned_tile(s, &tile);
    if (rc != IOLB_OK) return rc;
    // the one-kernel paths store the transformed kernels only
    const size_t bytes = tile.path == IOLB_PATH_FMA ? winograd_layout(C, (K + 31) / 32 * 32, m, 0, IOLB_PATH_FMA).total
                                                    : conv_winograd_workspace_bytes(N, C, H, W, K, m);
    DeviceState* dev = nullptr;
    rc = device_state(&dev);
    if (rc != IOLB_OK) return rc;
    void* ws = nullptr;
    rc = ensure_workspace(dev, bytes, &ws);
    if (rc != IOLB_OK) return rc;
    return run_winograd(x, w, nullptr, y, s, tile, ws, bytes);
}

int conv_winograd_pad(const float* x, const float* w, float* y, int N, int C, int H, int W, int K, int m, int pad)
{
    if (!x || !w || !y) return IOLB_EINVAL;
    iolb_shape s;
    int rc = make_wino_shape(N, C, H, W, K, m, &s, pad);
    if (rc != IOLB_OK) return rc;
    iolb_tile_config tile;
    rc = tuned_tile(s, &tile);
    if (rc != IOLB_OK) return rc;
    // workspace for the output extents of this padding
    const int P = H + 2 * pad - 2, Q = W + 2 * pad - 2;
    const int64_t tiles = (int64_t)N * ((P + m - 1) / m) * ((Q + m - 1) / m);
    const size_t bytes = tile.path == IOLB_PATH_FMA ? winograd_layout(C, (K + 31) / 32 * 32, m, 0, IOLB_PATH_FMA).total
                                                    : winograd_workspace_max(C, K, m, tiles);
    DeviceState* dev = nullptr;
    rc = device_state(&dev);
    if (rc != IOLB_OK) return rc;
    void* ws = nullptr;
    rc = ensure_workspace(dev, bytes, &ws);
    if (rc != IOLB_OK) return rc;
    return run_winograd(x, w, nullptr, y, s, tile, ws, bytes);
}

int iolb_winograd_matrices(int m, float* A, float* L, float* B)
{
    if (!A || !L || !B) return IOLB_EINVAL;
    auto copy = [&](auto mats) {
        using Mt = decltype(mats);
        constexpr int n = Mt::n;
        for (int i = 0; i < n - 2; ++i)
            for (int j = 0; j < n; ++j) A[i * n + j] = Mt::A[i][j];
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < 3; ++j) L[i * 3 + j] = Mt::L[i][j];
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) B[i * n + j] = Mt::B[i][j];
    };
    switch (m) {
    case 2: copy(iolb::Mats<2>{}); break;
    case 3: copy(iolb::Mats<3>{}); break;
    case 4: copy(iolb::Mats<4>{}); break;
    case 6: copy(iolb::Mats<6>{}); break;
    default: return IOLB_EUNSUPPORTED;
    }
    return IOLB_OK;
}

int iolb_set_stream(void* hip_stream)
{
    t_stream = static_cast<hipStream_t>(hip_stream);
    return IOLB_OK;
}

int iolb_timing_enable(int on)
{
    std::lock_guard<std::mutex> lock(g_mutex);
    g_timing = on != 0;
    return IOLB_OK;
}

int iolb_timing_read(int kind, int* launches, float* total_ms)
{
    if (!launches || !total_ms || kind < 0 || kind > 2) return IOLB_EINVAL;
    std::lock_guard<std::mutex> lock(g_mutex);
    float sum = 0.f;
    int count = 0;
    int rc = IOLB_OK;
    for (auto& ev : g_events[kind]) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(ev.second);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.first, ev.second);
        if (e != hipSuccess) rc = hip_fail(e);
        else { sum += ms; ++count; }
        hipEventDestroy(ev.first);
        hipEventDestroy(ev.second);
    }
    g_events[kind].clear();
    *launches = count;
    *total_ms = sum;
    return rc;
}

int iolb_probe_hbm_copy(const void* src, void* dst, size_t bytes, int reps, float* ms_per_launch)
{
    if (!src || !dst || !ms_per_launch || bytes == 0 || bytes % 16 || reps < 1) return IOLB_EINVAL;
    return time_probe(reps, ms_per_launch, [&] { return iolb::launch_probe_copy(src, dst, bytes, t_stream); });
}

size_t iolb_probe_mfma_sink_bytes(void)
{
    return sizeof(float) * 256 * (size_t)iolb::PROBE_MFMA_BLOCKS;
}

int iolb_probe_mfma_f32(void* sink, int iters, int reps, float* ms_per_launch, double* flop_per_launch)
{
    if (!sink || !ms_per_launch || !flop_per_launch || iters < 1 || reps < 1) return IOLB_EINVAL;
    *flop_per_launch = 4096.0 * iolb::PROBE_ACC * iters * 4.0 * iolb::PROBE_MFMA_BLOCKS;
    return time_probe(reps, ms_per_launch,
                      [&] { return iolb::launch_probe_mfma(static_cast<float*>(sink), iters, t_stream); });
}

size_t iolb_probe_share_scratch_bytes(void)
{
    return sizeof(unsigned long long) * 16 * (size_t)iolb::PROBE_SHARE_BLOCKS + 64;
}

int iolb_probe_pipeline_share(void* scratch, int slots, const int* roles, int iters, float* ms, double* ticks_per_slot)
{
    if (!scratch || !roles || !ms || !ticks_per_slot || slots < 1 || slots > 4 || iters < 1) return IOLB_EINVAL;
    unsigned packed = 0;
    for (int s = 0; s < slots; ++s) {
        if (roles[s] != IOLB_PROBE_ROLE_MFMA && roles[s] != IOLB_PROBE_ROLE_VALU) return IOLB_EINVAL;
        packed |= (unsigned)roles[s] << (2 * s);
    }
    auto* ticks = static_cast<unsigned long long*>(scratch);
    float* sink = reinterpret_cast<float*>(ticks + 16 * (size_t)iolb::PROBE_SHARE_BLOCKS);
    const int rc = time_probe(1, ms, [&] { return iolb::launch_probe_share(ticks, sink, slots, packed, iters, t_stream); });
    if (rc != IOLB_OK) return rc;
    std::vector<unsigned long long> host(16 * (size_t)iolb::PROBE_SHARE_BLOCKS);
    IOLB_HIP(hipMemcpyAsync(host.data(), ticks, host.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost, t_stream));
    IOLB_HIP(hipStreamSynchronize(t_stream));
    for (int s = 0; s < slots; ++s) {
        double sum = 0;
        for (int b = 0; b < iolb::PROBE_SHARE_BLOCKS; ++b)
            for (int w = 0; w < 4; ++w) sum += (double)host[(size_t)b * 16 + s * 4 + w];
        ticks_per_slot[s] = sum / (4.0 * iolb::PROBE_SHARE_BLOCKS);
    }
    return IOLB_OK;
}

int iolb_release_workspace(void)
{
    int dev = 0;
    IOLB_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_mutex);
    auto it = g_devices.find(dev);
    if (it == g_devices.end()) return IOLB_OK;
    DeviceState& d = it->second;
    if (d.ws.empty() && d.retired.empty()) return IOLB_OK;
    IOLB_HIP(hipDeviceSynchronize());          // nothing in flight may still use the buffers
    for (auto& kv : d.ws)
        if (kv.second.ptr) (void)hipFree(kv.second.ptr);
    for (void* p : d.retired) (void)hipFree(p);
    d.ws.clear();
    d.retired.clear();
    return IOLB_OK;
}

const char* iolb_strerror(int code)
{
    switch (code) {
    case IOLB_OK: return "success";
    case IOLB_EINVAL: return "invalid argument";
    case IOLB_EUNSUPPORTED: return "unsupported algorithm or Winograd tile size";
    case IOLB_ENOTILE: return "no tile fits the LDS / register budgets";
    case IOLB_EWORKSPACE: return "workspace missing, misaligned or too small";
    case IOLB_EHIP: return "HIP runtime error (see iolb_last_hip_error)";
    default: return "unknown error code";
    }
}

const char* iolb_last_hip_error(void) { return t_hip_error.c_str(); }

}  // extern "C"
