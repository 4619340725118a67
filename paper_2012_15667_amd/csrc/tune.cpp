// Host-side analytical tuner and lower-bound figures (no GPU code in this file).
//
// The searching domain is Table 1 of Sec. 6.2 read for a wave64 machine whose partial sums live in registers
// and whose staging buffers live in LDS.  Every tile carries two orders:
//   - `volume`: the paper's objective -- the reading volume of the dataflow of Sec. 5.2 (direct) / Sec. 5.3
//     (Winograd) evaluated exactly for the tile, ties by the distance from the optimality condition x y = R z.
//     iolb_tune_bound returns its minimum inside the optimality box.
//   - `key`: this build's own order, a modelled run time whose constants were fitted to tile sweeps on an
//     MI355X (a heuristic, not taken from the paper), with the reading volume as its memory term and
//     tie-break.  iolb_tune returns its minimum.
// All decisions are taken in 64-bit integers.
#include "iolbconv.h"
#include "tune.h"

#include <algorithm>
#include <array>
#include <cmath>
#include <cstdlib>
#include <vector>

namespace iolb {

namespace {

constexpr int64_t kComputeUnits = 256;   // grid-fill rule: a launch should keep every CU busy
constexpr int64_t kMaxThreads = 1024;    // largest workgroup: bounds the optimality box
constexpr int64_t kEffCap = 80;          // grid efficiency above this percentage is "good enough"
constexpr int64_t kLdsPerCu = 160 * 1024 - 256;   // LDS of a compute unit, minus a small reserve for alignment
constexpr int64_t kLdsHalf = 81920;      // "two blocks per multiprocessor" share (Sec. 6.2)

// LDS share of one workgroup when the caller gives none: half a compute unit's LDS, unless the tile's
// registers already limit the compute unit to one workgroup (then halving the LDS buys nothing).
int64_t auto_lds_budget(int threads, int acc)
{
    const int64_t waves_per_simd = std::max(threads / 256, 1);
    const bool two_fit = 2 * waves_per_simd * (acc + 64) <= 512;
    return two_fit ? kLdsHalf : kLdsPerCu;
}

std::vector<int> factors_of(int n) {
    std::vector<int> f;
    for (int d = 1; d <= n; ++d)
        if (n % d == 0) f.push_back(d);
    return f;
}

// Tile extents along an output axis of n pixels: the factors of n (Table 1) and, on the matrix-core path, the
// balanced cuts ceil(n / k) into k = 1..8 tiles, whose last tile hangs over the edge (its pixels past the
// image are computed on zeros and not stored) -- for extents with at most six factors (13, 28, 35, 55, 73,
// 147 ...), which leave too little choice; 56, 112 or 224 have enough.
std::vector<int> tile_extents(int n, bool ragged) {
    std::vector<int> e = factors_of(n);
    if (ragged && e.size() <= 6) {
        for (int k = 1; k <= 8; ++k) e.push_back((n + k - 1) / k);
        std::sort(e.begin(), e.end());
        e.erase(std::unique(e.begin(), e.end()), e.end());
    }
    return e;
}

bool allowed_threads(int64_t t) { return t == 64 || t == 128 || t == 256 || t == 512 || t == 1024; }

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Percentage of compute-unit slots busy over the rounds the grid needs, capped.
int64_t grid_efficiency(int64_t nblocks) {
    const int64_t rounds = ceil_div(nblocks, kComputeUnits);
    return std::min<int64_t>((100 * nblocks) / (rounds * kComputeUnits), kEffCap);
}

// Channels per stage: least zero-padding of C first, then the deepest stage that fits the LDS.
// bytes_per_channel covers `buffers` stage buffers; a stage that holds all C channels is the only one and
// needs a single buffer.
int choose_alpha(int C, const int* choices, int nchoices, int64_t bytes_per_channel, int64_t lds_bytes, int buffers = 1) {
    int best = 0;
    int64_t best_padded = 0;
    for (int i = 0; i < nchoices; ++i) {
        const int a = choices[i];
        if (bytes_per_channel * a / (a >= C ? buffers : 1) > lds_bytes) continue;
        if (a > 16 && ceil_div(C, a) < 4) continue;      // deep stages only where four or more remain to pipeline
        const int64_t padded = ceil_div(C, a) * a;
        if (best == 0 || padded < best_padded || (padded == best_padded && a > best)) {
            best = a;
            best_padded = padded;
        }
    }
    return best;
}

struct WaveGrid {
    int idle, threads, reads, wm, wn, acc;
    bool operator<(const WaveGrid& o) const {
        return std::array<int, 6>{idle, threads, reads, wm, wn, acc} <
               std::array<int, 6>{o.idle, o.threads, o.reads, o.wm, o.wn, o.acc};
    }
};

// Wave grids for MB x NB blocks of 32 x 32 partial sums: a wave owns mbw x nbw blocks (mbw in {1,2}, at most 8
// blocks = 128 accumulator registers); waves_m divides MB, waves_n = ceil(NB / nbw) -- the last wave column may
// own blocks past the tile, which stay idle.  One grid per workgroup size: the one with the fewest idle blocks,
// then the fewest operand reads.  Ascending in (idle, threads, ...): the first is the tightest fit.
std::vector<WaveGrid> wave_grids(int MB, int NB, int vgpr_budget, bool exact_only) {
    std::vector<WaveGrid> best;                       // at most one per thread count
    for (int wm = 1; wm <= MB; ++wm) {
        if (MB % wm) continue;
        const int mbw = MB / wm;
        if (mbw != 1 && mbw != 2) continue;
        for (int nbw = 1; nbw <= 8 && nbw <= NB; ++nbw) {
            if (mbw * nbw > 8) continue;
            const int wn = (NB + nbw - 1) / nbw;
            if (exact_only && wn * nbw != NB) continue;
            const int64_t threads = 64LL * wm * wn;
            if (!allowed_threads(threads) || 16 * mbw * nbw > vgpr_budget) continue;
            // a compute unit's register file holds 131072 lane-registers; leave 64 per lane for operands
            if (16 * mbw * nbw + 64 > 131072 / threads) continue;
            const WaveGrid g{wn * nbw - NB, (int)threads, mbw + nbw, wm, wn, 16 * mbw * nbw};
            bool placed = false;
            for (auto& o : best)
                if (o.threads == g.threads) {
                    if (g < o) o = g;
                    placed = true;
                }
            if (!placed) best.push_back(g);
        }
    }
    std::sort(best.begin(), best.end());
    return best;
}

// Modelled run time, in matrix-core clock cycles, of a direct-convolution tile on the MFMA path.  The
// structure follows the kernel: per stage a wave keeps its SIMD's matrix core busy for steps * blocks * 64
// cycles and also issues its operand reads (32 cycles each) and its share of the stage's load instructions
// (300 cycles each: a load rewrites the LDS base register and waits for the previous one); the waves of a
// workgroup that share a SIMD overlap these with each other's matrix work; workgroups run one per compute
// unit (several, if they have at most four waves) in rounds; the result cannot beat the time the reading and writing volumes need.  The constants were
// fitted to tile sweeps on an MI355X.  Integers only, so that both implementations of the tuner agree bit
// for bit.
// The model proper, shared by direct convolution and the Winograd product: a workgroup of `waves` waves, each
// owning mbw x nbw blocks, runs `stages` stages of `steps` MFMA steps and `loads` load instructions per wave.
int64_t block_cost(int64_t steps, int64_t mbw, int64_t nbw, int64_t loads, int64_t waves, int64_t acc, int64_t lds_used,
                   int64_t stages, int64_t nblocks, int64_t memory_cycles) {
    const int64_t mfma = steps * mbw * nbw * 64;                 // cycles one wave's stage keeps the matrix core busy
    const int64_t own = mfma + steps * (mbw + nbw) * 32 + 300 * loads;
    // Workgroups of up to four waves leave room on their compute unit, so several are resident at once: as many
    // as the LDS holds and the registers hold (512 per SIMD lane, acc + 64 per wave), at most 4 one-wave or 2
    // larger workgroups, and no more than the layer has per compute unit.  Waves of different workgroups overlap
    // a little less well than those of one (+10 % on the shared matrix-core time).  Larger workgroups are
    // modelled one per compute unit.
    int64_t resident = 1;
    if (waves <= 4)
        resident = std::max<int64_t>(1, std::min({kLdsPerCu / lds_used, 4 * (512 / (acc + 64)) / waves,
                                                  (int64_t)(waves == 1 ? 4 : 2), ceil_div(nblocks, kComputeUnits)}));
    const int64_t sharing = ceil_div(resident * waves, 4);       // waves per SIMD
    // what the waves of a SIMD cannot hide from each other: their matrix-core time, and 8 cycles of it per operand
    // read (the reads of one wave hold up the MFMA issue of the others)
    const int64_t per_wave = mfma + steps * (mbw + nbw) * 8;
    const int64_t shared = resident > 1 ? per_wave * sharing * 11 / 10 : per_wave * sharing;
    const int64_t stage = (sharing > 1 ? std::max(shared, own) : own) + 100 * waves;           // + barrier
    const int64_t workgroup = stages * stage + 15000 + 200 * acc;                              // + start-up, stores
    const int64_t compute = ceil_div(nblocks, kComputeUnits * resident) * workgroup;
    return std::max(compute, memory_cycles);
}

int64_t mfma_tile_cost(const iolb_shape& s, int b, int x, int y, int z, int alpha, const WaveGrid& g,
                       int64_t nblocks, int64_t q_read, int64_t q_write) {
    const int64_t RS = (int64_t)s.R * s.S;
    const int64_t waves = g.threads / 64;
    const int64_t mbw = (z / 32) / g.wm, nbw = g.acc / 16 / mbw;
    const int64_t xh = (int64_t)(x - 1) * s.stride + s.S, yh = (int64_t)(y - 1) * s.stride + s.R;
    const int64_t halo = b * xh * yh;
    // load instructions a wave issues per stage: input tile (flat chunks of 64 elements when a wave owns at
    // most 8 of them, else one per tile row and 64-column segment) per channel, plus its share of the weights
    const int64_t chunks_per_wave = ceil_div(ceil_div(halo, 64), waves);
    const int64_t loads_in = (chunks_per_wave <= 8 ? chunks_per_wave : ceil_div(b * yh * ceil_div(xh, 64), waves)) * alpha;
    const int64_t loads_w = ceil_div((int64_t)alpha * RS * (z / 4), 64 * waves);
    const int64_t lds_used = (alpha >= s.C ? 4 : 8) * alpha * (halo + RS * z);
    // bytes over bytes per cycle; a tile row shorter than 128 bytes still costs a whole 128-byte request
    const int64_t in_bytes = nblocks * s.C * b * yh * std::max<int64_t>(4 * xh, 128);
    const int64_t w_bytes = 4 * (q_read - nblocks * s.C * halo);
    const int64_t memory = (in_bytes + w_bytes) / 4000 + (4 * q_write) / 1500;
    return block_cost((alpha / 2) * RS, mbw, nbw, loads_in + loads_w, waves, g.acc, lds_used, ceil_div(s.C, alpha), nblocks, memory);
}

// The same model for a block of the unfused Winograd product: tb sub-domains by z channels of one plane, alpha
// rows of U (z floats) and of V (tb floats) per stage in 16-byte loads, one MFMA step per channel pair.
int64_t product_tile_cost(const iolb_shape& s, int64_t tb, int z, int alpha, const WaveGrid& g, int64_t nblocks,
                          int64_t q_read, int64_t m_elems) {
    const int64_t waves = g.threads / 64;
    const int64_t mbw = (z / 32) / g.wm, nbw = g.acc / 16 / mbw;
    const int64_t loads = ceil_div((int64_t)alpha * (z / 4), 64 * waves) + ceil_div((int64_t)alpha * (tb / 4), 64 * waves);
    const int64_t lds_used = (alpha >= s.C ? 4 : 8) * alpha * (tb + z);
    const int64_t memory = (4 * q_read) / 4000 + (4 * m_elems) / 1500;
    return block_cost(alpha / 2, mbw, nbw, loads, waves, g.acc, lds_used, ceil_div(s.C, alpha), nblocks, memory);
}

int pow2_at_least(int v) {
    int p = 1;
    while (p < v) p *= 2;
    return p;
}

void direct_candidates(const iolb_shape& s, int P, int Q, int64_t lds_bytes, int vgpr_budget, int path,
                       bool use_box, std::vector<Candidate>* out) {
    static const int alphas_mfma[] = {64, 32, 16, 8, 4};       // whole channel quads: two per lane half
    static const int alphas_fma[] = {16, 8, 4, 2, 1};
    const int64_t box = kMaxThreads * vgpr_budget;
    const int64_t RS = (int64_t)s.R * s.S, st2 = (int64_t)s.stride * s.stride;
    // matrix-core path: z runs over the factors of K rounded up to whole 32-channel blocks (the channels
    // past K are computed as zeros and not stored)
    const int Kz = path == IOLB_PATH_MFMA ? (s.K + 31) / 32 * 32 : s.K;
    const auto fb = factors_of(s.N), fz = factors_of(Kz);
    const auto fx = tile_extents(Q, path == IOLB_PATH_MFMA), fy = tile_extents(P, path == IOLB_PATH_MFMA);
    for (int b : fb)
        for (int x : fx)
            for (int y : fy) {
                const int64_t npix = (int64_t)b * x * y;
                const int64_t xh = (int64_t)(x - 1) * s.stride + s.S, yh = (int64_t)(y - 1) * s.stride + s.R;
                const int64_t halo = b * xh * yh;
                for (int z : fz) {
                    if (use_box && !((int64_t)z * z * RS <= box * st2 && npix * npix * st2 <= box * RS)) continue;
                    const int64_t per_stage = halo + RS * z;
                    std::vector<WaveGrid> grids;
                    if (path == IOLB_PATH_MFMA) {
                        if (z % 32) continue;
                        // the tightest wave grid, and the larger workgroups that idle on at most a quarter of the
                        // tile's blocks more: more waves per SIMD hide the loads of small layers
                        const int NB = (int)((npix + 31) / 32);
                        for (const WaveGrid& g : wave_grids(z / 32, NB, vgpr_budget, false))
                            if (grids.empty() || 4 * (g.idle - grids.front().idle) <= NB) grids.push_back(g);
                    } else {
                        if (npix > 256) continue;
                        const int lanes = std::max(pow2_at_least((int)npix), 16);
                        for (int T : {64, 128, 256}) {
                            if (lanes > T) continue;
                            const int groups = T / lanes;
                            if (z % groups) continue;
                            const int per_thread = z / groups;
                            if (per_thread > 16 || per_thread > vgpr_budget) continue;
                            grids.push_back(WaveGrid{0, T, 0, groups, 1, per_thread});
                            break;               // ascending T: the first is the smallest
                        }
                    }
                    for (const WaveGrid& g : grids) {
                        int alpha = 0;
                        int lds_mult = 0;
                        if (path == IOLB_PATH_MFMA) {
                            alpha = choose_alpha(s.C, alphas_mfma, 5, 8 * per_stage,
                                                 lds_bytes ? lds_bytes : auto_lds_budget(g.threads, g.acc), 2);
                            // automatic budget: a stage too large for half the LDS (large kernels) may take all of
                            // it, as long as the smallest weight slab (4 channels, 32 kernels) leaves half to the
                            // input tile
                            if (alpha == 0 && !lds_bytes && 8 * 4 * RS * 32 <= kLdsPerCu / 2)
                                alpha = choose_alpha(s.C, alphas_mfma, 5, 8 * per_stage, kLdsPerCu, 2);
                            lds_mult = alpha >= s.C ? 4 : 8;            // one stage only: one buffer
                        } else {
                            alpha = choose_alpha(s.C, alphas_fma, 5, 4 * per_stage, lds_bytes ? lds_bytes : kLdsHalf);
                            lds_mult = 4;
                        }
                        if (alpha == 0) continue;
                        const int64_t nblocks = (int64_t)(s.N / b) * ceil_div(Q, x) * ceil_div(P, y) * (Kz / z);
                        Candidate c{};
                        c.cfg.b = b; c.cfg.x = x; c.cfg.y = y; c.cfg.z = z;
                        c.cfg.alpha = alpha;
                        c.cfg.threads = g.threads; c.cfg.waves_m = g.wm; c.cfg.waves_n = g.wn;
                        c.cfg.path = path; c.cfg.wt_mode = 0;
                        c.cfg.lds_bytes_used = (int32_t)(lds_mult * alpha * per_stage);
                        c.cfg.acc_regs_per_thread = g.acc;
                        c.cfg.q_read_elems = nblocks * s.C * per_stage;
                        c.cfg.q_write_elems = (int64_t)s.N * s.K * P * Q;
                        c.volume = {c.cfg.q_read_elems, std::llabs(npix * st2 - RS * z), -npix * z, -(int64_t)x, z, b, y, g.threads, -path, 0};
                        if (path == IOLB_PATH_MFMA) {
                            const int64_t cost = mfma_tile_cost(s, b, x, y, z, alpha, g, nblocks, c.cfg.q_read_elems,
                                                                c.cfg.q_write_elems);
                            c.key = {cost, c.cfg.q_read_elems, -npix * z, -(int64_t)x, z, b, y, g.threads, 0, 0};
                        } else {
                            c.key = {-grid_efficiency(nblocks), 0, c.cfg.q_read_elems, std::llabs(npix * st2 - RS * z),
                                     -npix * z, -(int64_t)x, z, b, y, g.threads};
                        }
                        out->push_back(c);
                    }
                }
            }
}

// 1 x 1 convolution, no padding (any stride: output pixel (p, q) reads input pixel (stride p, stride q) only): the
// pixels of an image do not interact, so the output plane is one row of P Q pixels and a workgroup of pointwise_mfma.hip covers four waves' ranges of 32 nbw consecutive pixels of that
// row (x = 128 nbw pixels, y = 1; the ranges of a workgroup may lie in neighbouring images) by z = 32 mbw output
// channels.  Each entry of kPointShapes is a wave shape the kernel is instantiated for, with stages of 16
// channels, or 32 where that pads no channel.  Reading volume: per workgroup and channel x inputs and z weights.
// In this build's order these tiles come before the general ones (measured 1.3 to 2.4 times faster on every
// 1 x 1 layer of the networks timed), ranked among themselves by a modelled time: the waves are dealt over 1024
// SIMDs; a SIMD runs its waves' MFMAs one after the other (64 cycles each) and hides all but one wave's other
// work (40 cycles per step of loads and address arithmetic) behind them; the result cannot beat the time the
// memory traffic needs (same rates as for the general tiles; the inputs count once, because the channel blocks of
// one pixel range run next to each other on one XCD and find them in its L2).
struct PointShape { int mbw, nbw; };
constexpr PointShape kPointShapes[] = {{1, 1}, {1, 2}, {1, 4}, {2, 2}, {2, 4}};

bool pointwise_layer(const iolb_shape& s) {
    return s.algo == IOLB_DIRECT && s.R == 1 && s.S == 1 && s.pad == 0 &&
           4LL * s.C * s.H * s.W < (1LL << 32);          // a lane's byte offset inside its image is 32 bits
}

void pointwise_candidates(const iolb_shape& s, int P, int Q, int vgpr_budget, bool use_box, std::vector<Candidate>* out) {
    const int64_t box = kMaxThreads * vgpr_budget;
    const int64_t HW = (int64_t)P * Q;
    for (const PointShape& w : kPointShapes)
        for (int alpha : {16, 32}) {
            if (alpha == 32 && s.C % 32) continue;
            const int64_t z = 32 * w.mbw, npix = 128 * w.nbw, acc = 16 * w.mbw * w.nbw;
            if (use_box && !(z * z <= box && npix * npix <= box)) continue;
            if (acc > vgpr_budget) continue;
            const int64_t nbk = ceil_div(s.K, z);
            const int64_t nwaves = (int64_t)s.N * ceil_div(HW, 32 * w.nbw);
            const int64_t nblocks = ceil_div(nwaves, 4) * nbk;
            Candidate c{};
            c.cfg.b = 1; c.cfg.x = (int32_t)npix; c.cfg.y = 1; c.cfg.z = (int32_t)z;
            c.cfg.alpha = alpha;
            c.cfg.threads = 256; c.cfg.waves_m = 1; c.cfg.waves_n = 4;
            c.cfg.path = IOLB_PATH_POINT; c.cfg.wt_mode = 0;
            c.cfg.lds_bytes_used = (int32_t)(8 * alpha * z);
            c.cfg.acc_regs_per_thread = (int32_t)acc;
            c.cfg.q_read_elems = nblocks * s.C * (npix + z);
            c.cfg.q_write_elems = (int64_t)s.N * s.K * P * Q;
            const int64_t steps = ceil_div(s.C, alpha) * alpha / 2;
            const int64_t compute = ceil_div(nwaves * nbk, 1024) * steps * w.mbw * w.nbw * 64 + steps * 40 + 15000;
            // (with a stride the rows between the output rows are never touched, the pixels between the output
            // pixels come along in the same memory lines)
            const int64_t memory = (4 * ((int64_t)s.N * s.C * HW * s.stride + nblocks * s.C * z)) / 4000 + (4 * c.cfg.q_write_elems) / 1500;
            const int64_t cost = std::max(compute, memory);
            // ties: bound by memory, the smaller block (more waves, more loads in flight); else the smaller volume
            c.key = {-(1LL << 61), cost, memory >= compute ? npix * z : 0, c.cfg.q_read_elems, -npix * z, z, -alpha, 0, 0, 0};
            c.volume = {c.cfg.q_read_elems, std::llabs(npix - z), -npix * z, -npix, z, 1, 1, 256, -IOLB_PATH_POINT, alpha};
            out->push_back(c);
        }
}

// Thin layers in direct convolution (3 x 3 kernels, stride 1, at most four input channels; direct_thin.hip): a lane
// owns tw neighbouring output pixels of a row (tw = 4 when the rows are whole quads, else 1) and every output
// channel, with its 3 x (tw + 2) input window of all C channels in registers; a workgroup is 256 such lanes in
// (image, row, column) order.  Reported as b = 1, x = 256 tw, y = 1, z = K, alpha = C, path FMA, wt_mode 2.
// Reading volume, counted as if every workgroup were one strip of a row: C (3 (x + 2) + 9 K) per workgroup.  In
// this build's order it comes before every other tile (measured: such layers are bound by their stores, and this
// kernel is the one that overlaps them with its arithmetic); in the paper's order it competes by volume.
bool thin_direct_layer(const iolb_shape& s) {
    return s.algo == IOLB_DIRECT && s.R == 3 && s.S == 3 && s.stride == 1 && s.C <= 4;
}

void thin_direct_candidates(const iolb_shape& s, int P, int Q, int vgpr_budget, std::vector<Candidate>* out) {
    const int tw = Q % 4 == 0 ? 4 : 1;
    if (s.C * 3 * (tw + 2) > vgpr_budget) return;
    const int64_t x = 256 * tw;
    const int64_t nblocks = ceil_div((int64_t)s.N * P * ceil_div(Q, tw), 256);
    Candidate c{};
    c.cfg.b = 1; c.cfg.x = (int32_t)x; c.cfg.y = 1; c.cfg.z = s.K;
    c.cfg.alpha = s.C;
    c.cfg.threads = 256; c.cfg.waves_m = 1; c.cfg.waves_n = 4;
    c.cfg.path = IOLB_PATH_FMA; c.cfg.wt_mode = 2;
    c.cfg.lds_bytes_used = 0;
    c.cfg.acc_regs_per_thread = tw;
    c.cfg.q_read_elems = nblocks * s.C * (3 * (x + 2) + 9 * (int64_t)s.K);
    c.cfg.q_write_elems = (int64_t)s.N * s.K * P * Q;
    c.key = {-(1LL << 62), 0, c.cfg.q_read_elems, 0, 0, s.K, 256, 0, 0, 0};
    c.volume = {c.cfg.q_read_elems, std::llabs(x - 9 * (int64_t)s.K), -x * s.K, -x, s.K, 1, 1, 256, 0, 2};
    out->push_back(c);
}

// Winograd: the resident block is tb sub-domains by z output channels of ONE transformed plane
// (the channel-summation temporaries of step 3); per channel it reads tb transformed inputs and
// z transformed weights, for each of the (m+2)^2 planes.
// The fused matrix-core blocks of wino_fused_mfma.hip: every plane of a tb x z block resident in accumulator
// registers (Sec. 5.3).  Each entry is one kernel instantiation.
struct FusedBlock { int m, tb, z, alpha, threads, waves_m, waves_n, lds_bytes, acc; };
constexpr FusedBlock kFusedBlocks[] = {
    {2, 64, 64, 8, 1024, 8, 2, 131072, 64},     // F(2x2): 2 x 2 blocks of 32 x 32, four row waves each
    {4, 32, 64, 4, 768, 12, 1, 148480, 96},     // F(4x4): 1 x 2 blocks, six row waves each
};

void winograd_candidates(const iolb_shape& s, int P, int Q, int m, int64_t lds_bytes, int vgpr_budget, bool auto_regs,
                         bool use_box, std::vector<Candidate>* out) {
    static const int alphas[] = {16, 8, 4};
    const int64_t planes = (int64_t)(m + 2) * (m + 2);
    const int64_t tiles = (int64_t)s.N * ceil_div(P, m) * ceil_div(Q, m);
    const int64_t box = kMaxThreads * vgpr_budget;
    const int64_t top = std::min<int64_t>(ceil_div(tiles, 32) * 32, 1024);
    const int Kz = (s.K + 31) / 32 * 32;        // whole 32-channel blocks; the channels past K are zeros
    // Thin layers: the (m+2)^2 transformed values of all C channels of a sub-domain fit in one lane's
    // registers, so the four steps run in one kernel (the fused dataflow of Sec. 5.3): a workgroup of 256
    // lanes covers 256 sub-domains and every output channel, reads its input windows and the transformed
    // kernels once and writes the outputs -- no temporaries in memory.  Ranked before every unfused tile:
    // those move (m+2)^2 / m^2 times the output tensor to memory and back.
    if (s.C <= 4 && planes * s.C <= vgpr_budget) {
        const int64_t nblocks = ceil_div(tiles, 256);
        Candidate c{};
        c.cfg.b = 1; c.cfg.x = (int32_t)(m * 256); c.cfg.y = m; c.cfg.z = Kz;
        c.cfg.alpha = s.C;
        c.cfg.threads = 256; c.cfg.waves_m = 1; c.cfg.waves_n = 4;
        c.cfg.path = IOLB_PATH_FMA; c.cfg.wt_mode = 1;
        c.cfg.lds_bytes_used = 0;
        c.cfg.acc_regs_per_thread = (int32_t)(planes * s.C);
        c.cfg.q_read_elems = nblocks * s.C * planes * (256 + Kz);
        c.cfg.q_write_elems = (int64_t)s.N * s.K * P * Q;
        c.key = {-(1LL << 62), 0, c.cfg.q_read_elems, 0, 0, Kz, 256, 0, 0, 0};
        c.volume = {-(1LL << 62), 0, 0, 0, Kz, 256, 0, 0, 0, 0};
        out->push_back(c);
    }
    // Fused matrix-core blocks, for any channel count: per channel a block reads the input windows of its tb
    // sub-domains (a strip of m tb + 2 by m + 2 pixels) and (m+2)^2 z transformed weights, and nothing else: this
    // is the dataflow of Sec. 5.3, so in the paper's order (`volume`) they come before the unfused tiles, whose
    // transformed inputs and products make a round trip through memory that q_read does not show.  In this
    // build's order a fused block comes first only where a time model says it beats the unfused path (heuristic;
    // constants measured on an MI355X, in nanoseconds):
    //   unfused: product flop at 105 Tflop/s + (x + V + M + y) bytes at 5.2 TB/s + 4 launches of 3 us;
    //   fused:   rounds of 256 workgroups, each its own flop at the rate of one compute unit (370 flop/ns for
    //            F(2x2), 295 for F(4x4)) + 2 launches.
    {
        const int64_t Cp16 = ceil_div(s.C, 16) * 16;
        const int64_t tiles_p = ceil_div(tiles, 32) * 32;
        const int64_t flop_unfused = 2 * planes * tiles_p * Cp16 * Kz;
        const int64_t bytes_unfused = 4 * ((int64_t)s.N * s.C * s.H * s.W + planes * tiles_p * (Cp16 + Kz) + (int64_t)s.N * s.K * P * Q);
        const int64_t t_unfused = flop_unfused / 105000 + bytes_unfused / 5200 + 4 * 3000;
        for (const FusedBlock& f : kFusedBlocks) {
            if (f.m != m) continue;
            if (lds_bytes && f.lds_bytes > lds_bytes) continue;
            if (!auto_regs && f.acc > vgpr_budget) continue;
            // the kernels address a block's windows with byte offsets below 2^30 from the block's first image; a
            // block of tb sub-domains touches at most tb / (sub-domains per image) + 2 images
            const int64_t tpi = (int64_t)ceil_div(P, m) * ceil_div(Q, m);
            if ((ceil_div(f.tb, tpi) + 2) * (int64_t)s.C * s.H * s.W * 4 >= (1LL << 30)) continue;
            const int64_t Kf = ceil_div(s.K, f.z) * f.z, Cf = ceil_div(s.C, f.alpha) * f.alpha;
            const int64_t nblocks = ceil_div(tiles, f.tb) * (Kf / f.z);
            const int64_t t_fused = ceil_div(nblocks, kComputeUnits) * (2 * planes * f.tb * f.z * Cf / (m == 2 ? 370 : 295)) + 2 * 3000;
            Candidate c{};
            c.cfg.b = 1; c.cfg.x = m * f.tb; c.cfg.y = m; c.cfg.z = f.z;
            c.cfg.alpha = f.alpha;
            c.cfg.threads = f.threads; c.cfg.waves_m = f.waves_m; c.cfg.waves_n = f.waves_n;
            c.cfg.path = IOLB_PATH_FUSED; c.cfg.wt_mode = 1;
            c.cfg.lds_bytes_used = f.lds_bytes;
            c.cfg.acc_regs_per_thread = f.acc;
            c.cfg.q_read_elems = nblocks * s.C * ((int64_t)(m * f.tb + 2) * (m + 2) + planes * f.z);
            c.cfg.q_write_elems = (int64_t)s.N * s.K * P * Q;
            c.key = {t_fused < t_unfused ? -(1LL << 61) : 1, 0, c.cfg.q_read_elems, 0, 0, f.z, f.threads, f.alpha, 0, 0};
            c.volume = {-(1LL << 61), c.cfg.q_read_elems, 0, 0, f.z, f.threads, 0, 0, 0, 0};
            out->push_back(c);
        }
    }
    const auto fz = factors_of(Kz);
    for (int64_t tb = 32; tb <= top; tb += 32)
        for (int z : fz) {
            if (z % 32) continue;
            if (use_box && !((int64_t)z * z <= box && tb * tb <= box)) continue;
            for (const WaveGrid& g : wave_grids(z / 32, (int)(tb / 32), vgpr_budget, true)) {    // tb is free: no idle blocks
                const int alpha = choose_alpha(s.C, alphas, 3, 8 * (tb + z),
                                               lds_bytes ? lds_bytes : auto_lds_budget(g.threads, g.acc), 2);
                if (alpha == 0) continue;
                const int64_t ntb = ceil_div(tiles, tb);
                const int64_t nblocks = planes * ntb * (Kz / z);
                Candidate c{};
                c.cfg.b = 1; c.cfg.x = (int32_t)(m * tb); c.cfg.y = m; c.cfg.z = z;
                c.cfg.alpha = alpha;
                c.cfg.threads = g.threads; c.cfg.waves_m = g.wm; c.cfg.waves_n = g.wn;
                c.cfg.path = IOLB_PATH_MFMA; c.cfg.wt_mode = 1;
                c.cfg.lds_bytes_used = (int32_t)((alpha >= s.C ? 4 : 8) * alpha * (tb + z));     // one stage only: one buffer
                c.cfg.acc_regs_per_thread = g.acc;
                c.cfg.q_read_elems = nblocks * s.C * (tb + z);
                c.cfg.q_write_elems = (int64_t)s.N * s.K * P * Q;
                const int64_t cost = product_tile_cost(s, tb, z, alpha, g, nblocks, c.cfg.q_read_elems, planes * Kz * ntb * tb);
                c.key = {0, cost, c.cfg.q_read_elems, std::llabs(tb - z), -tb * z, z, g.threads, 0, 0, 0};
                c.volume = {0, c.cfg.q_read_elems, std::llabs(tb - z), -tb * z, z, g.threads, 0, 0, 0, 0};
                out->push_back(c);
            }
        }
}

}  // namespace

int winograd_m(int algo) {
    switch (algo) {
    case IOLB_WINO_F2: return 2;
    case IOLB_WINO_F3: return 3;
    case IOLB_WINO_F4: return 4;
    case IOLB_WINO_F6: return 6;
    default: return 0;
    }
}

int validate_shape(const iolb_shape& s, int* P, int* Q) {
    if (s.N < 1 || s.C < 1 || s.H < 1 || s.W < 1 || s.K < 1 || s.R < 1 || s.S < 1 || s.stride < 1 || s.pad < 0)
        return IOLB_EINVAL;
    if (s.algo != IOLB_DIRECT && winograd_m(s.algo) == 0) return IOLB_EUNSUPPORTED;
    if (s.algo != IOLB_DIRECT && (s.R != 3 || s.S != 3 || s.stride != 1)) return IOLB_EUNSUPPORTED;
    if ((int64_t)s.H + 2LL * s.pad < s.R || (int64_t)s.W + 2LL * s.pad < s.S) return IOLB_EINVAL;
    const int64_t p = ((int64_t)s.H + 2LL * s.pad - s.R) / s.stride + 1;
    const int64_t q = ((int64_t)s.W + 2LL * s.pad - s.S) / s.stride + 1;
    // tensors of up to 2^31 - 1 elements each
    if ((int64_t)s.N * s.C * s.H * s.W >= (1LL << 31) || (int64_t)s.N * s.K * p * q >= (1LL << 31) ||
        (int64_t)s.K * s.C * s.R * s.S >= (1LL << 31)) return IOLB_EINVAL;
    *P = (int)p;
    *Q = (int)q;
    return IOLB_OK;
}

int enumerate_fma(const iolb_shape& s, int64_t lds_bytes, int vgpr_budget, std::vector<Candidate>* out) {
    int P = 0, Q = 0;
    const int rc = validate_shape(s, &P, &Q);
    if (rc != IOLB_OK) return rc;
    out->clear();
    if (s.algo != IOLB_DIRECT) return IOLB_OK;
    direct_candidates(s, P, Q, std::max<int64_t>(lds_bytes, 0), vgpr_budget > 0 ? vgpr_budget : 128, IOLB_PATH_FMA, false, out);
    std::sort(out->begin(), out->end(), [](const Candidate& a, const Candidate& b) { return a.key < b.key; });
    return IOLB_OK;
}

int enumerate(const iolb_shape& s, int64_t lds_bytes, int vgpr_budget, bool use_box, std::vector<Candidate>* out) {
    int P = 0, Q = 0;
    const int rc = validate_shape(s, &P, &Q);
    if (rc != IOLB_OK) return rc;
    if (lds_bytes < 0) lds_bytes = 0;       // 0: per-tile automatic budget
    const bool auto_regs = vgpr_budget <= 0;
    if (vgpr_budget <= 0) vgpr_budget = 128;
    out->clear();
    if (s.algo == IOLB_DIRECT) {
        direct_candidates(s, P, Q, lds_bytes, vgpr_budget, IOLB_PATH_MFMA, use_box, out);
        // The plain-FMA path serves when no matrix-core tile fits, and also when none of them covers two
        // blocks of 32 pixels: very large kernels, whose weight slab leaves the LDS room for a few pixels only
        // (an 11 x 11, stride-4 first layer: at most 25 pixels per tile; 0.59 ms on the best matrix-core tile,
        // 0.27 ms on the FMA path).  FMA tiles carry no modelled time; their keys start below zero and sort
        // first.
        int64_t most_pixels = 0;
        for (const auto& c : *out) most_pixels = std::max<int64_t>(most_pixels, (int64_t)c.cfg.b * c.cfg.x * c.cfg.y);
        const bool fma = most_pixels < 64;
        if (fma) direct_candidates(s, P, Q, lds_bytes, vgpr_budget, IOLB_PATH_FMA, use_box, out);
        if (pointwise_layer(s)) pointwise_candidates(s, P, Q, vgpr_budget, use_box, out);
        if (thin_direct_layer(s)) thin_direct_candidates(s, P, Q, vgpr_budget, out);
    } else {
        winograd_candidates(s, P, Q, winograd_m(s.algo), lds_bytes, vgpr_budget, auto_regs, use_box, out);
    }
    std::sort(out->begin(), out->end(), [](const Candidate& a, const Candidate& b) { return a.key < b.key; });
    return IOLB_OK;
}

int tune(const iolb_shape& s, int64_t lds_bytes, int vgpr_budget, iolb_tile_config* cfg) {
    std::vector<Candidate> c;
    // Direct convolution: the modelled time ranks the whole domain (the optimality box stays available to
    // iolb_enumerate as the pruning device of the measured search).  Winograd: box first.
    int rc = enumerate(s, lds_bytes, vgpr_budget, s.algo != IOLB_DIRECT, &c);
    if (rc != IOLB_OK) return rc;
    bool any_unfused = false;
    for (const auto& cand : c) any_unfused = any_unfused || cand.cfg.path != IOLB_PATH_FUSED;
    if (!any_unfused) {                    // tiny layers: no unfused tile inside the box, search the whole domain
        rc = enumerate(s, lds_bytes, vgpr_budget, false, &c);
        if (rc != IOLB_OK) return rc;
    }
    if (c.empty()) return IOLB_ENOTILE;
    *cfg = c.front().cfg;
    return IOLB_OK;
}

int tune_by_volume(const iolb_shape& s, int64_t lds_bytes, int vgpr_budget, iolb_tile_config* cfg) {
    std::vector<Candidate> c;
    int rc = enumerate(s, lds_bytes, vgpr_budget, true, &c);
    if (rc != IOLB_OK) return rc;
    if (c.empty()) {                       // tiny layers: nothing inside the box, search the whole domain
        rc = enumerate(s, lds_bytes, vgpr_budget, false, &c);
        if (rc != IOLB_OK) return rc;
    }
    if (c.empty()) return IOLB_ENOTILE;
    const Candidate* best = &c.front();
    for (const auto& cand : c)
        if (cand.volume < best->volume) best = &cand;
    *cfg = best->cfg;
    return IOLB_OK;
}

// ---------------------------------------------------------------------------------------
// lower-bound figures (Sec. 4 and Sec. 5), in double precision
// ---------------------------------------------------------------------------------------
int bounds(const iolb_shape& s, int64_t Sf, iolb_bounds_out* o) {
    int P = 0, Q = 0;
    const int rc = validate_shape(s, &P, &Q);
    if (rc != IOLB_OK) return rc;
    if (Sf < 1) return IOLB_EINVAL;
    const double npq = (double)s.N * P * Q;
    o->P = P;
    o->Q = Q;
    o->q_write_elems = (int64_t)s.N * s.K * P * Q;
    o->compulsory_elems = (int64_t)s.N * s.C * s.H * s.W + (int64_t)s.K * s.C * s.R * s.S + o->q_write_elems;
    const double S = (double)Sf;
    if (s.algo == IOLB_DIRECT) {
        const double RS = (double)s.R * s.S;
        const double reuse = RS / ((double)s.stride * s.stride);      // Eq. "definition of R"
        o->vertices = (2LL * s.R * s.S * s.C - 1) * (int64_t)s.N * P * Q * s.K;
        const double S2 = 2.0 * S;
        o->t_bound_2s = 4.0 * S2 * std::sqrt(reuse * S2) + S2 - 1.0;
        o->q_lower_lead = RS * s.C * npq * s.K / (4.0 * std::sqrt(2.0 * reuse * S));
        o->q_lower_explicit = S * ((double)o->vertices / o->t_bound_2s - 1.0);
        o->q_dataflow = 2.0 * npq * s.K * RS * s.C / std::sqrt(reuse * S) + npq * s.K;
    } else {
        const int m = winograd_m(s.algo);
        const int64_t n = m + 2, n2 = n * n, r = 3;
        const int64_t tiles = (int64_t)s.N * ceil_div(P, m) * ceil_div(Q, m);
        const int64_t per_tile_k = (2 * n2 - 1) * n2 * s.C + (2 * r * r - 1) * n2 * s.C + n2 * s.C +
                                   (int64_t)(s.C - 1) * n2 + (2 * n2 - 1) * m * m;
        o->vertices = tiles * s.K * per_tile_k;
        const double S2 = 2.0 * S;
        const double er = (double)m * r;
        o->t_bound_2s = 2.0 * (double)(n * n * n) / er * S2 * std::sqrt(S2) + 6.0 * (double)n2 / er * S2;
        o->q_lower_lead = npq * s.K * s.C * (double)n * r / (m * std::sqrt(S));
        const double v_lead = 2.0 * npq * s.K * s.C * (double)(n2 * n2) / ((double)m * m);
        o->q_lower_explicit = S * (v_lead / o->t_bound_2s - 1.0);
        o->q_dataflow = 2.0 * npq * s.K * s.C * r * (double)n / (m * std::sqrt(S)) + npq * s.K;
    }
    return IOLB_OK;
}

}  // namespace iolb

extern "C" int iolb_tune(const iolb_shape* shape, size_t lds_bytes, int vgpr_budget, iolb_tile_config* out) {
    if (!shape || !out || vgpr_budget < 0) return IOLB_EINVAL;
    return iolb::tune(*shape, (int64_t)lds_bytes, vgpr_budget, out);
}

extern "C" int iolb_tune_bound(const iolb_shape* shape, size_t lds_bytes, int vgpr_budget, iolb_tile_config* out) {
    if (!shape || !out || vgpr_budget < 0) return IOLB_EINVAL;
    return iolb::tune_by_volume(*shape, (int64_t)lds_bytes, vgpr_budget, out);
}

extern "C" int64_t iolb_enumerate(const iolb_shape* shape, size_t lds_bytes, int vgpr_budget, int use_box,
                                  iolb_tile_config* out, int64_t capacity) {
    if (!shape || vgpr_budget < 0 || capacity < 0) return IOLB_EINVAL;
    std::vector<iolb::Candidate> c;
    const int rc = iolb::enumerate(*shape, (int64_t)lds_bytes, vgpr_budget, use_box != 0, &c);
    if (rc != IOLB_OK) return rc;
    if (out)
        for (int64_t i = 0; i < (int64_t)c.size() && i < capacity; ++i) out[i] = c[i].cfg;
    return (int64_t)c.size();
}

extern "C" int iolb_bounds(const iolb_shape* shape, int64_t S_f_elems, iolb_bounds_out* out) {
    if (!shape || !out) return IOLB_EINVAL;
    return iolb::bounds(*shape, S_f_elems, out);
}
