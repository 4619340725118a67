"""TEST INFRASTRUCTURE ONLY: exact evaluation of the paper's I/O-bound expressions and of the
tile-selection rule, in Python integers and rationals.

Every function cites the passage it evaluates.  Quantities that contain a square root are
returned as floats computed from an exact rational radicand; everything the GPU library's
tuner is compared with bit-for-bit is an integer.

Notation (paper -> here): W_ker,H_ker -> S,R (kernel width,height); C_in -> C; C_out -> K;
W_out,H_out -> Q,P; mu -> stride; the paper's reuse number "R" -> rho; the paper's fast-memory
size "S" -> Sf (elements); e -> e (Winograd output tile edge); r -> r.  A batch of N images
(absent from the paper's formulas) multiplies the output plane: W_out*H_out -> N*P*Q.
No code is shared with the GPU library.
"""
from fractions import Fraction
from math import isqrt, sqrt

DIRECT, WINO_F2, WINO_F4, WINO_F3, WINO_F6 = 0, 1, 2, 3, 4
WINO_E = {WINO_F2: 2, WINO_F3: 3, WINO_F4: 4, WINO_F6: 6}     # output tile extent e of each Winograd algo id
PATH_FMA, PATH_MFMA, PATH_FUSED, PATH_POINT = 0, 1, 2, 3

# ------------------------------------------------------------------------------------------
# shapes
# ------------------------------------------------------------------------------------------

def out_extent(H, W, R, S, stride, pad):
    return (H + 2 * pad - R) // stride + 1, (W + 2 * pad - S) // stride + 1


def rho(R, S, stride):
    """Maximum number of sliding windows that reuse one input element (Sec. 4.2, Eq. 'definition of R')."""
    return Fraction(R * S, stride * stride)


# ------------------------------------------------------------------------------------------
# vertex counts
# ------------------------------------------------------------------------------------------

def summation_tree(k):
    """(internal, output) vertices of a summation tree with k inputs (Sec. 4.2, first lemma)."""
    return (k - 2 if k >= 2 else 0, 1)


def linear_combination_tree(k):
    """(internal, output) vertices of a linear-combination tree with k inputs (Sec. 4.3, first
    lemma): k products plus the k-2 internal sums of a summation tree."""
    return (k + summation_tree(k)[0], 1)


def V_DC(N, C, P, Q, K, R, S):
    """Internal + output vertices of the direct-convolution DAG (Sec. 4.2, second lemma)."""
    return (2 * R * S * C - 1) * P * Q * K * N


def V_WA_steps(C, e, r=3):
    """Per (tile, output channel) vertex counts of the four Winograd steps, as the proof of the
    vertex-count lemma of Sec. 4.3 lists them.  Returns a dict of integers."""
    n = e + r - 1
    return {
        "input_transform": (2 * n * n - 1) * n * n * C,
        "kernel_transform": (2 * r * r - 1) * n * n * C,
        "products": n * n * C,
        "channel_sums": (C - 1) * n * n,
        "output_transform": (2 * n * n - 1) * e * e,
    }


def V_WA_lead(N, C, P, Q, K, e, r=3):
    """Leading term of the Winograd vertex count, 2 W_out H_out C_out C_in (e+r-1)^4 / e^2."""
    n = e + r - 1
    return Fraction(2 * N * P * Q * K * C * n ** 4, e * e)


# ------------------------------------------------------------------------------------------
# T(S) bounds and lower bounds
# ------------------------------------------------------------------------------------------

def _sqrt_fraction(fr):
    fr = Fraction(fr)
    num, den = fr.numerator, fr.denominator
    rn, rd = isqrt(num), isqrt(den)
    if rn * rn == num and rd * rd == den:
        return Fraction(rn, rd)          # exact when the radicand is a perfect square
    return sqrt(num / den)


def T_DC(Sf, rho_):
    """Upper bound on a partition subset, T(S) <= 4 S sqrt(rho S) + S - 1 (Sec. 4.2, third lemma)."""
    return 4 * Sf * _sqrt_fraction(rho_ * Sf) + Sf - 1


def general_lower_bound(V, T_2S, Sf):
    """Q >= S (|V| / T(2S) - 1)  (Sec. 4.1, theorem 'general I/O lower bound')."""
    return Sf * (V / T_2S - 1)


def Qlow_DC_explicit(N, C, P, Q, K, R, S, stride, Sf):
    """The general bound with the direct-convolution vertex count and T bound substituted:
    V / (8 sqrt(2 rho S) + 2 - 1/S) - S.   (The proof of the direct-convolution theorem prints
    the trailing term as 1/S; carrying out the substitution gives S.)"""
    root = _sqrt_fraction(2 * rho(R, S, stride) * Sf)
    return V_DC(N, C, P, Q, K, R, S) / (8 * root + 2 - Fraction(1, Sf)) - Sf


def Qlow_DC_lead(N, C, P, Q, K, R, S, stride, Sf):
    """Leading term W_ker H_ker C_in W_out H_out C_out / (4 sqrt(2 rho S))  (Sec. 4.2 theorem)."""
    return (R * S * C * P * Q * K * N) / (4 * _sqrt_fraction(2 * rho(R, S, stride) * Sf))


def T_WA(Sf, e, r=3):
    """T(S) = 2 (e+r-1)^3/(e r) S sqrt(S) + 6 (e+r-1)^2/(e r) S  (Sec. 4.3, T lemma)."""
    n = e + r - 1
    return Fraction(2 * n ** 3, e * r) * Sf * _sqrt_fraction(Sf) + Fraction(6 * n * n, e * r) * Sf


def Qlow_WA_lead(N, C, P, Q, K, e, Sf, r=3):
    """W_out H_out C_out C_in (e+r-1) r / (e sqrt(S))  (Sec. 4.3 theorem, as printed)."""
    n = e + r - 1
    return Fraction(N * P * Q * K * C * n * r, e) / _sqrt_fraction(Sf)


# ------------------------------------------------------------------------------------------
# dataflow I/O volumes (Sec. 5)
# ------------------------------------------------------------------------------------------

def Qread_DC_paper(C, P, Q, K, R, S, stride, x, y, z):
    """(H_out W_out C_out / xyz) * H_ker W_ker C_in (z + xy/rho)   (Sec. 5.2, first display)."""
    return Fraction(P * Q * K, x * y * z) * R * S * C * (z + Fraction(x * y) / rho(R, S, stride))


def Qread_DC_min(C, P, Q, K, R, S, stride, xyz):
    """Its lower envelope 2 H W C_out H_ker W_ker C_in sqrt(1/(rho xyz)), reached iff xy = rho z."""
    return 2 * P * Q * K * R * S * C * _sqrt_fraction(1 / (rho(R, S, stride) * xyz))


def Qread_WA_paper(C, P, Q, K, x, y, z, r=3):
    """(H_out W_out C_out / xyz) * (xy C_in + z r^2 C_in)   (Sec. 5.3, first display)."""
    return Fraction(P * Q * K, x * y * z) * (x * y * C + z * r * r * C)


def Qread_WA_min(C, P, Q, K, xyz, r=3):
    """Its lower envelope 2 r H W C_out C_in / sqrt(xyz), reached iff xy = r^2 z."""
    return 2 * r * P * Q * K * C / _sqrt_fraction(xyz)


def Q_DC_total(C, P, Q, K, R, S, stride, Sf, Np=1):
    """2 H W C_out H_ker W_ker C_in / sqrt(rho S / N_p) + H W C_out   (Sec. 5.2, Eq. 'Q of actual DC')."""
    return 2 * P * Q * K * R * S * C / _sqrt_fraction(rho(R, S, stride) * Fraction(Sf, Np)) + P * Q * K


def Q_WA_total(C, P, Q, K, e, Sf, Np=1, r=3):
    """2 H W C_out C_in r (e+r-1) / (e sqrt(S/N_p)) + H W C_out   (Sec. 5.3, last display)."""
    n = e + r - 1
    return Fraction(2 * P * Q * K * C * r * n, e) / _sqrt_fraction(Fraction(Sf, Np)) + P * Q * K


def compulsory(N, C, H, W, K, R, S, P, Q):
    """Every input and weight loaded once, every output stored once (Sec. 3.1)."""
    return N * C * H * W + K * C * R * S + N * K * P * Q


def bounds(shape, Sf):
    """The figures the library's iolb_bounds reports, for comparison.  shape is a dict with
    N,C,H,W,K,R,S,stride,pad,algo."""
    s = shape
    P, Q = out_extent(s["H"], s["W"], s["R"], s["S"], s["stride"], s["pad"])
    out = {"P": P, "Q": Q,
           "compulsory_elems": compulsory(s["N"], s["C"], s["H"], s["W"], s["K"], s["R"], s["S"], P, Q),
           "q_write_elems": s["N"] * s["K"] * P * Q}
    if s["algo"] == DIRECT:
        r_ = rho(s["R"], s["S"], s["stride"])
        out["vertices"] = V_DC(s["N"], s["C"], P, Q, s["K"], s["R"], s["S"])
        out["t_bound_2s"] = float(T_DC(2 * Sf, r_))
        out["q_lower_lead"] = float(Qlow_DC_lead(s["N"], s["C"], P, Q, s["K"], s["R"], s["S"], s["stride"], Sf))
        out["q_lower_explicit"] = float(Qlow_DC_explicit(s["N"], s["C"], P, Q, s["K"], s["R"], s["S"], s["stride"], Sf))
        out["q_dataflow"] = float(Q_DC_total(s["C"], s["N"] * P, Q, s["K"], s["R"], s["S"], s["stride"], Sf))
    else:
        e = WINO_E[s["algo"]]
        steps = V_WA_steps(s["C"], e)
        tiles = s["N"] * (-(-P // e)) * (-(-Q // e))
        out["vertices"] = tiles * s["K"] * sum(steps.values())
        out["t_bound_2s"] = float(T_WA(2 * Sf, e))
        out["q_lower_lead"] = float(Qlow_WA_lead(s["N"], s["C"], P, Q, s["K"], e, Sf))
        out["q_lower_explicit"] = float(general_lower_bound(V_WA_lead(s["N"], s["C"], P, Q, s["K"], e),
                                                            T_WA(2 * Sf, e), Sf))
        out["q_dataflow"] = float(Q_WA_total(s["C"], s["N"] * P, Q, s["K"], e, Sf))
    return out


# ------------------------------------------------------------------------------------------
# the paper's tile rule: searching domain of Table 1 (Sec. 6.2), objective of Sec. 5.2
# ------------------------------------------------------------------------------------------
#
# Everything in this section follows the paper alone (with the batch reading: a block covers b images).  The
# library's bound-only pick (iolb_tune_bound) applies the same order to the tiles its kernels can run.

def input_tile(x, y, R, S, stride):
    """Extents x', y' of the input tile under an x by y output block: the paper approximates x' ~ mu x
    (Sec. 5.2); exactly, x' = mu (x - 1) + W_ker."""
    return (x - 1) * stride + S, (y - 1) * stride + R


def Qread_exact(N, C, P, Q, K, R, S, stride, b, x, y, z):
    """Reading volume of the dataflow of Sec. 5.2 for an output block of b images, x by y pixels and z
    channels: every block loads, per input channel, its b x' y' input tile and the W_ker H_ker z weights of its
    z kernels, once.  Blocks that hang over an edge count whole."""
    xp, yp = input_tile(x, y, R, S, stride)
    nblocks = (N // b) * (-(-Q // x)) * (-(-P // y)) * (-(-K // z))
    return nblocks * C * (b * xp * yp + R * S * z)


def in_optimality_box(b, x, y, z, R, S, stride, Sb):
    """Table 1: z <= sqrt(S_b / rho) and x y <= sqrt(S_b rho), rho = W_ker H_ker / mu^2, in integers."""
    return z * z * R * S <= Sb * stride * stride and (b * x * y) ** 2 * stride * stride <= Sb * R * S


def paper_domain(N, P, Q, K, R, S, stride, Sb, z_step=1):
    """Table 1: tile extents are factors of the output extents (b | N for the batch), the block fits the fast
    memory of a processor, b x y z <= S_b, and lies inside the optimality box.  z_step: granularity of z the
    hardware asks for (1: none)."""
    out = []
    for b in divisors(N):
        for x in divisors(Q):
            for y in divisors(P):
                for z in divisors(K):
                    if z % z_step == 0 and b * x * y * z <= Sb and in_optimality_box(b, x, y, z, R, S, stride, Sb):
                        out.append((b, x, y, z))
    return out


def volume_order(N, C, P, Q, K, R, S, stride, b, x, y, z):
    """The order of the bound-only rule: reading volume; then the distance from the optimality condition
    b x y = rho z (Sec. 5.2, in integers: |b x y mu^2 - W_ker H_ker z|); then the fuller block (the dataflow
    wants x y z ~ S / N_p); then the longer rows, fewer channels, fewer images."""
    return (Qread_exact(N, C, P, Q, K, R, S, stride, b, x, y, z),
            abs(b * x * y * stride * stride - R * S * z), -b * x * y * z, -x, z, b, y)


def tune_by_volume(N, C, P, Q, K, R, S, stride, Sb, z_step=1):
    """(b, x, y, z) of least reading volume in the paper's domain, or None when the domain is empty."""
    dom = paper_domain(N, P, Q, K, R, S, stride, Sb, z_step)
    if not dom:
        return None
    return min(dom, key=lambda t: volume_order(N, C, P, Q, K, R, S, stride, *t))


# ------------------------------------------------------------------------------------------
# tile selection (the analytical tuner)
# ------------------------------------------------------------------------------------------
#
# The searching domain is Table 1 of Sec. 6.2 read for a wave64 machine whose partial sums live
# in registers and whose staging buffers live in LDS:
#   * tile extents are factors of the output extents (b | N, x | W_out, y | H_out, z | C_out);
#   * the resident output block must fit the accumulator registers of the workgroup,
#     b x y z <= T * vgpr_budget                                   ("xyz <= S_b");
#   * the optimality condition xy = rho z bounds the box:  z <= sqrt(S_b/rho), xy <= sqrt(S_b rho),
#     with S_b the largest workgroup's accumulator capacity, 1024 * vgpr_budget;
#   * the per-stage input tile x' * y' * alpha and the weight slab R S alpha z, double buffered,
#     must fit lds_bytes (the LDS share of one workgroup; when 0, S_sm / 2, or S_sm if the tile's
#     registers allow only one workgroup per compute unit anyway).
# Two orders over the same tiles:
#   * bound_pick: the paper's order (volume_order above) -- what the library's iolb_tune_bound returns;
#   * tune: THIS BUILD'S HEURISTIC, not the paper's: among feasible matrix-core tiles it minimises a modelled run
#     time (mfma_tile_cost) in which the read volume is the memory term and the tie-break; FMA-path tiles keep
#     a simpler order (grid fill, then read volume); a fused Winograd block comes first where fused_faster says
#     so.  The constants of the model are listed in MODEL_CONSTANTS with the measurement each came from; they
#     are mirrored from the library, so the bit-for-bit comparison of `tune` with iolb_tune checks that two
#     implementations agree, not that the heuristic is right ("parity unpinned" for tune, candidates,
#     mfma_tile_cost, _wave_grids, _pick_alpha, _auto_lds_budget, fused_faster).

MODEL_CONSTANTS = {
    # name: (value, unit, where it came from)
    "operand_read": (32, "cycles per LDS operand read of a wave", "fit to 300-tile sweeps on 21 layers, one MI355X"),
    "operand_read_shared": (8, "cycles of a SIMD's matrix-core time per operand read of any of its waves",
                            "250-tile sweeps with several wave grids per tile on cfg3, cfg5a-d, AlexNet conv2/3"),
    "load_issue": (300, "cycles per LDS-direct load instruction", "s_memtime around the issue of back-to-back loads"),
    "barrier": (100, "cycles per wave and stage", "fit to the same sweeps"),
    "startup": (15000, "cycles per workgroup", "fit to the same sweeps"),
    "store": (200, "cycles per accumulator register", "fit to the same sweeps"),
    "read_rate": (4000, "bytes per cycle, whole chip", "fit; the streaming-copy probe reads 2000-2700"),
    "write_rate": (1500, "bytes per cycle, whole chip", "fit; the streaming-copy probe writes 1900-2300"),
    "resident_penalty": (11, "tenths: matrix time of several resident workgroups", "150-tile sweeps on 19 layers"),
    "unfused_flop_rate": (105000, "flop per ns, Winograd product kernel", "bench step, eight layers"),
    "transform_rate": (5200, "bytes per ns, Winograd transform kernels", "cfg5c transforms, rocprofv3 durations"),
    "launch": (3000, "ns per kernel launch", "cfg2, back-to-back launches"),
    "fused_rate": ({2: 370, 4: 295}, "flop per ns and compute unit, fused Winograd kernels", "cfg5b-d, 95 / 75 Tflop/s"),
}

N_CU = 256
T_MAX = 1024
LDS_CU = 160 * 1024 - 256      # LDS of a compute unit, minus a small reserve for alignment
REGS_PER_LANE = 512            # registers per lane of a SIMD (4 SIMDs x 64 lanes x 512 = 131072 per CU)


def _auto_lds_budget(T, acc):
    """LDS share of one workgroup when the caller gives none: half a compute unit's LDS (two blocks
    per multiprocessor, Sec. 6.2) -- unless the tile's registers already limit the compute unit to one
    workgroup, in which case halving the LDS would buy nothing and the whole LDS is used."""
    waves_per_simd = max(T // 256, 1)
    two_fit = 2 * waves_per_simd * (acc + 64) <= REGS_PER_LANE
    return 81920 if two_fit else LDS_CU

T_CHOICES = (64, 128, 256, 512, 1024)
EFF_CAP = 80


def divisors(n):
    return [d for d in range(1, n + 1) if n % d == 0]


def _grid_efficiency_pct(nblocks):
    rounds = -(-nblocks // N_CU)
    return min((100 * nblocks) // (rounds * N_CU), EFF_CAP)


def _pick_alpha(C, choices, per_alpha_bytes, lds_bytes, buffers=1):
    """Channels per stage: least channel padding first, then the deepest stage that fits (stages of 32 or 64
    channels, which help 1x1 kernels whose stages are short, only where at least four stages remain).  per_alpha_bytes
    covers `buffers` stage buffers; a stage that holds all C channels is the only one and needs one."""
    best = None
    for a in choices:
        if per_alpha_bytes * a // (buffers if a >= C else 1) > lds_bytes:
            continue
        if a > 16 and -(-C // a) < 4:          # deep stages only where four or more remain to pipeline
            continue
        padded = -(-C // a) * a
        key = (padded, -a)
        if best is None or key < best[0]:
            best = (key, a)
    return None if best is None else best[1]


def _wave_grids(MB, NB, vgpr_budget, exact_only=False):
    """Wave grids for MB x NB blocks of 32 x 32 outputs: a wave owns mbw x nbw blocks (mbw in {1,2}, at most 8
    blocks); waves_m divides MB, waves_n = ceil(NB / nbw) -- the last wave column may own blocks past the tile,
    which stay idle.  One grid per workgroup size (fewest idle blocks, then fewest operand reads), ascending in
    (idle blocks, threads, ...): the first is the tightest fit."""
    best = {}
    for wm in divisors(MB):
        mbw = MB // wm
        if mbw not in (1, 2):
            continue
        for nbw in range(1, 9):
            if mbw * nbw > 8 or nbw > NB:
                continue
            wn = -(-NB // nbw)
            if exact_only and wn * nbw != NB:
                continue
            T = 64 * wm * wn
            if T not in T_CHOICES:
                continue
            if 16 * mbw * nbw > vgpr_budget:
                continue
            if 16 * mbw * nbw + 64 > 131072 // T:      # register-file share of a lane, 64 kept for operands
                continue
            g = (wn * nbw - NB, T, mbw + nbw, wm, wn, 16 * mbw * nbw)
            if T not in best or g < best[T]:
                best[T] = g
    return sorted(best.values())


def _cdiv(a, b):
    return -(-a // b)


def block_cost(steps, mbw, nbw, loads, waves, acc, lds_used, stages, nblocks, memory_cycles):
    """The model proper (matrix-core clock cycles), shared by direct convolution and the Winograd product: a
    workgroup of `waves` waves, each owning mbw x nbw blocks of 32 x 32 partial sums, runs `stages` stages of
    `steps` MFMA steps (64 cycles per block) and `loads` load instructions per wave (300 cycles each), plus 32
    cycles per operand read; waves that share a SIMD hide that behind each other's matrix work; a barrier costs
    100 cycles per wave; a workgroup pays 15000 cycles to start and 200 per accumulator register to store.
    Workgroups of up to four waves leave room on their compute unit, so several are resident at once: as many
    as the LDS and the registers hold (512 per SIMD lane, acc + 64 per wave), at most 4 one-wave or 2 larger
    ones, no more than the layer has per compute unit; waves of different workgroups overlap a little less
    well (+10 % on the shared matrix-core time).  Rounds over the 256 compute units; never below the time the
    memory traffic needs.  See MODEL_CONSTANTS for where the numbers come from."""
    mfma = steps * mbw * nbw * 64
    own = mfma + steps * (mbw + nbw) * 32 + 300 * loads
    resident = 1
    if waves <= 4:
        resident = max(1, min(LDS_CU // lds_used, 4 * (512 // (acc + 64)) // waves, 4 if waves == 1 else 2,
                              _cdiv(nblocks, N_CU)))
    sharing = _cdiv(resident * waves, 4)                    # waves per SIMD
    per_wave = mfma + steps * (mbw + nbw) * 8               # operand reads hold up the MFMA issue of the SIMD's other waves
    shared = per_wave * sharing * 11 // 10 if resident > 1 else per_wave * sharing
    stage = (max(shared, own) if sharing > 1 else own) + 100 * waves
    workgroup = stages * stage + 15000 + 200 * acc
    compute = _cdiv(nblocks, N_CU * resident) * workgroup
    return max(compute, memory_cycles)


def mfma_tile_cost(s, b, x, y, z, alpha, T, wm, acc, nblocks, q_read, q_write):
    """Modelled run time of a direct-convolution tile on the matrix-core path: the ranking function of this
    build's tile rule.  steps = alpha/2 * R*S per stage; load instructions per wave and stage: the input tile in
    flat chunks of 64 elements when a wave owns at most 8 of them (else one per tile row and 64 columns), per
    channel, plus its share of the weight slab in 16-byte pieces.  Memory floor: reads at 4000 and writes at 1500
    bytes per cycle, a tile row counting at least one 128-byte request."""
    RS = s["R"] * s["S"]
    waves = T // 64
    mbw = (z // 32) // wm
    nbw = acc // 16 // mbw
    xp, yp = (x - 1) * s["stride"] + s["S"], (y - 1) * s["stride"] + s["R"]
    halo = b * xp * yp
    chunks_per_wave = _cdiv(_cdiv(halo, 64), waves)
    if chunks_per_wave <= 8:
        loads_in = chunks_per_wave * alpha                              # 64-element chunks of the flat tile
    else:
        loads_in = _cdiv(b * yp * _cdiv(xp, 64), waves) * alpha         # one per tile row and 64 columns
    loads_w = _cdiv(alpha * RS * (z // 4), 64 * waves)
    lds_used = (4 if alpha >= s["C"] else 8) * alpha * (halo + RS * z)
    in_bytes = nblocks * s["C"] * b * yp * max(4 * xp, 128)     # a short tile row still costs a 128-byte request
    w_bytes = 4 * (q_read - nblocks * s["C"] * halo)
    memory = (in_bytes + w_bytes) // 4000 + (4 * q_write) // 1500
    return block_cost((alpha // 2) * RS, mbw, nbw, loads_in + loads_w, waves, acc, lds_used, _cdiv(s["C"], alpha),
                      nblocks, memory)


def product_tile_cost(s, tb, z, alpha, T, wm, acc, nblocks, q_read, m_elems):
    """The same model for a block of the unfused Winograd product: tb sub-domains by z channels of one plane, alpha
    rows of U (z floats) and of V (tb floats) per stage in 16-byte loads, one MFMA step per channel pair."""
    waves = T // 64
    mbw = (z // 32) // wm
    nbw = acc // 16 // mbw
    loads = _cdiv(alpha * (z // 4), 64 * waves) + _cdiv(alpha * (tb // 4), 64 * waves)
    lds_used = (4 if alpha >= s["C"] else 8) * alpha * (tb + z)
    memory = (4 * q_read) // 4000 + (4 * m_elems) // 1500
    return block_cost(alpha // 2, mbw, nbw, loads, waves, acc, lds_used, _cdiv(s["C"], alpha), nblocks, memory)


def _pow2ceil(v):
    p = 1
    while p < v:
        p *= 2
    return p


def tile_extents(n, path):
    """Tile extents along an output axis of n pixels: the factors of n (Table 1) and, on the matrix-core path,
    the balanced cuts ceil(n / k) into k = 1..8 tiles, whose last tile hangs over the edge (its pixels past
    the image are computed on zeros and not stored) -- for extents with at most six factors (13, 28, 35, 55,
    73, 147 ...), which leave too little choice; 56, 112 or 224 have enough."""
    ext = set(divisors(n))
    if path == PATH_MFMA and len(ext) <= 6:
        ext |= {-(-n // k) for k in range(1, 9)}
    return sorted(ext)


def _direct_candidates(s, P, Q, lds_bytes, vgpr_budget, path, use_f3):
    N, C, K, R, S, st = s["N"], s["C"], s["K"], s["R"], s["S"], s["stride"]
    sb_max = T_MAX * vgpr_budget
    cands = []
    # matrix-core path: z divides K rounded up to whole 32-channel blocks (channels past K: zeros, not stored)
    Kz = -(-K // 32) * 32 if path == PATH_MFMA else K
    for b in divisors(N):
        for x in tile_extents(Q, path):
            for y in tile_extents(P, path):
                npix = b * x * y
                xp, yp = (x - 1) * st + S, (y - 1) * st + R
                halo = b * xp * yp
                for z in divisors(Kz):
                    if use_f3 and not (z * z * R * S <= sb_max * st * st and
                                       npix * npix * st * st <= sb_max * R * S):
                        continue
                    if path == PATH_MFMA:
                        if z % 32:
                            continue
                        # the tightest wave grid, and the larger workgroups that idle on at most a quarter of the
                        # tile's blocks more
                        NB = -(-npix // 32)
                        grids = []
                        for g in _wave_grids(z // 32, NB, vgpr_budget):
                            if not grids or 4 * (g[0] - grids[0][0]) <= NB:
                                grids.append(g)
                    else:
                        if npix > 256:
                            continue
                        PL = max(_pow2ceil(npix), 16)
                        grids = []
                        for T in (64, 128, 256):
                            if PL > T:
                                continue
                            KG = T // PL
                            if z % KG or z // KG > 16 or z // KG > vgpr_budget:
                                continue
                            grids.append((0, T, 0, KG, 1, z // KG))
                            break
                    for _, T, _, wm, wn, acc in grids:
                        if path == PATH_MFMA:
                            budget = lds_bytes if lds_bytes else _auto_lds_budget(T, acc)
                            alpha = _pick_alpha(C, (64, 32, 16, 8, 4), 8 * (halo + R * S * z), budget, 2)
                            # a stage too large for half the LDS (large kernels) may take all of it, provided the
                            # smallest weight slab (4 channels of 32 kernels, two buffers) leaves half to the tile
                            if alpha is None and not lds_bytes and 8 * 4 * R * S * 32 <= LDS_CU // 2:
                                alpha = _pick_alpha(C, (64, 32, 16, 8, 4), 8 * (halo + R * S * z), LDS_CU, 2)
                            lds_mult = 4 if alpha is not None and alpha >= C else 8      # one stage only: one buffer
                        else:
                            alpha = _pick_alpha(C, (16, 8, 4, 2, 1), 4 * (halo + R * S * z), lds_bytes or 81920)
                            lds_mult = 4
                        if alpha is None:
                            continue
                        nblocks = (N // b) * (-(-Q // x)) * (-(-P // y)) * (Kz // z)
                        qread = nblocks * C * (halo + R * S * z)
                        if path == PATH_MFMA:
                            cost = mfma_tile_cost(s, b, x, y, z, alpha, T, wm, acc, nblocks, qread, N * K * P * Q)
                            key = (cost, qread, -npix * z, -x, z, b, y, T, 0, 0)
                        else:
                            key = (-_grid_efficiency_pct(nblocks), 0, qread, abs(npix * st * st - R * S * z),
                                   -npix * z, -x, z, b, y, T)
                        cands.append((key, dict(b=b, x=x, y=y, z=z, alpha=alpha, threads=T, waves_m=wm,
                                                waves_n=wn, path=path, wt_mode=0,
                                                lds_bytes_used=lds_mult * alpha * (halo + R * S * z),
                                                acc_regs_per_thread=acc, q_read_elems=qread,
                                                q_write_elems=N * K * P * Q)))
    return cands


# 1 x 1 convolution, no padding (any stride: an output pixel reads one input pixel): the pixels of an image do not
# interact, so the output plane is one row of P Q pixels.  A workgroup of the library's kernel for these layers is four waves, each on 32 nbw consecutive pixels of
# that row (x = 128 nbw, y = 1; a workgroup may run on into the next image) by z = 32 mbw output channels; stages of
# 16 channels, or 32 where that pads none.  POINT_SHAPES: the (mbw, nbw) the kernel is instantiated for.
POINT_SHAPES = ((1, 1), (1, 2), (1, 4), (2, 2), (2, 4))


def pointwise_layer(s):
    return (s["algo"] == DIRECT and s["R"] == 1 and s["S"] == 1 and s["pad"] == 0
            and 4 * s["C"] * s["H"] * s["W"] < (1 << 32))


def pointwise_read_volume(N, C, HW, K, x, z):
    """Reading volume of the dataflow of Sec. 5.2 for R = S = 1 on the row of HW pixels per image: every block of x
    pixels (made of four ranges of x / 4, dealt image after image) by z channels reads, per input channel, its x
    inputs and z weights."""
    ranges = N * _cdiv(HW, x // 4)
    return _cdiv(ranges, 4) * _cdiv(K, z) * C * (x + z)


def _pointwise_candidates(s, P, Q, vgpr_budget, use_f3):
    """THIS BUILD'S HEURISTIC for the order among these tiles (modelled time: the waves dealt over 1024 SIMDs, a SIMD
    runs its waves' MFMAs one after the other, 64 cycles each, and hides all but one wave's 40 cycles per step of
    other work; never faster than the memory traffic allows, the inputs counted once because the channel blocks of
    a pixel range share them through L2) and for ranking them before the general tiles (measured)."""
    N, C, K = s["N"], s["C"], s["K"]
    HW = P * Q
    sb_max = T_MAX * vgpr_budget
    cands = []
    for mbw, nbw in POINT_SHAPES:
        for alpha in (16, 32):
            if alpha == 32 and C % 32:
                continue
            z, npix, acc = 32 * mbw, 128 * nbw, 16 * mbw * nbw
            if use_f3 and not (z * z <= sb_max and npix * npix <= sb_max):
                continue
            if acc > vgpr_budget:
                continue
            nbk = _cdiv(K, z)
            nwaves = N * _cdiv(HW, 32 * nbw)
            qread = pointwise_read_volume(N, C, HW, K, npix, z)
            qwrite = N * K * P * Q
            steps = _cdiv(C, alpha) * alpha // 2
            compute = _cdiv(nwaves * nbk, 1024) * steps * mbw * nbw * 64 + steps * 40 + 15000
            nblocks = _cdiv(nwaves, 4) * nbk
            memory = (4 * (N * C * HW * s["stride"] + nblocks * C * z)) // 4000 + (4 * qwrite) // 1500
            cost = max(compute, memory)
            # ties: bound by memory, the smaller block (more waves, more loads in flight); else the smaller volume
            key = (-(1 << 61), cost, npix * z if memory >= compute else 0, qread, -npix * z, z, -alpha, 0, 0, 0)
            cands.append((key, dict(b=1, x=npix, y=1, z=z, alpha=alpha, threads=256, waves_m=1, waves_n=4,
                                    path=PATH_POINT, wt_mode=0, lds_bytes_used=8 * alpha * z,
                                    acc_regs_per_thread=acc, q_read_elems=qread, q_write_elems=qwrite)))
    return cands


def thin_direct_layer(s):
    return s["algo"] == DIRECT and s["R"] == 3 and s["S"] == 3 and s["stride"] == 1 and s["C"] <= 4


def _thin_direct_candidates(s, P, Q, vgpr_budget):
    """Thin layers in direct convolution: a lane owns tw neighbouring output pixels of a row (4 when the rows are
    whole quads, else 1) and every output channel, its 3 x (tw + 2) input window of all C channels in registers; a
    workgroup is 256 such lanes.  Reading volume counted as if every workgroup were one strip of a row.  Ranked
    before every other tile in this build's order (heuristic, measured)."""
    N, C, K = s["N"], s["C"], s["K"]
    tw = 4 if Q % 4 == 0 else 1
    if C * 3 * (tw + 2) > vgpr_budget:
        return []
    x = 256 * tw
    nblocks = _cdiv(N * P * _cdiv(Q, tw), 256)
    qread = nblocks * C * (3 * (x + 2) + 9 * K)
    key = (-(1 << 62), 0, qread, 0, 0, K, 256, 0, 0, 0)
    return [(key, dict(b=1, x=x, y=1, z=K, alpha=C, threads=256, waves_m=1, waves_n=4, path=PATH_FMA, wt_mode=2,
                       lds_bytes_used=0, acc_regs_per_thread=tw, q_read_elems=qread, q_write_elems=N * K * P * Q))]


# Fused matrix-core blocks (every plane of a tb x z block resident in accumulator registers, Sec. 5.3), one per
# kernel instantiation of the library: (e, tb, z, alpha, threads, waves_m, waves_n, lds_bytes, acc)
FUSED_BLOCKS = (
    (2, 64, 64, 8, 1024, 8, 2, 131072, 64),
    (4, 32, 64, 4, 768, 12, 1, 148480, 96),
)


def fused_faster(s, P, Q, e, ftb, fz, falpha):
    """Heuristic of this build (integers, nanoseconds): does the fused block beat the unfused path?
    unfused: product flop at 105 Tflop/s + (x + V + M + y) bytes at 5.2 TB/s + 4 launches of 3 us;
    fused: rounds of 256 workgroups, each its own flop at one compute unit's rate, + 2 launches."""
    N, C, K = s["N"], s["C"], s["K"]
    n2 = (e + 2) * (e + 2)
    tiles = N * (-(-P // e)) * (-(-Q // e))
    Kz, Cp16, tiles_p = -(-K // 32) * 32, -(-C // 16) * 16, -(-tiles // 32) * 32
    t_unfused = (2 * n2 * tiles_p * Cp16 * Kz) // 105000 + \
                (4 * (N * C * s["H"] * s["W"] + n2 * tiles_p * (Cp16 + Kz) + N * K * P * Q)) // 5200 + 4 * 3000
    Cf = -(-C // falpha) * falpha
    nblocks = (-(-tiles // ftb)) * (-(-K // fz))
    t_fused = (-(-nblocks // N_CU)) * ((2 * n2 * ftb * fz * Cf) // (370 if e == 2 else 295)) + 2 * 3000
    return t_fused < t_unfused


def _wino_candidates(s, P, Q, e, lds_bytes, vgpr_budget, use_f3, auto_regs=True):
    """Winograd: the resident block is one transformed plane of `tb` sub-domains by z output
    channels (the channel-summation temporaries of step 3); per channel it reads tb transformed
    inputs and z transformed weights, for each of the (e+r-1)^2 planes.  Reported as a strip of
    tb sub-domains: b = 1, x = e * tb, y = e."""
    N, C, K = s["N"], s["C"], s["K"]
    n2 = (e + 2) * (e + 2)
    tiles = N * (-(-P // e)) * (-(-Q // e))
    sb_max = T_MAX * vgpr_budget
    cands = []
    tb_top = -(-tiles // 32) * 32
    Kz = -(-K // 32) * 32          # whole 32-channel blocks; the channels past K are zeros
    # Thin layers: all (e+2)^2 transformed values of every channel of a sub-domain fit in one lane's
    # registers, so the fused dataflow of Sec. 5.3 runs as one kernel (256 sub-domains per workgroup, every
    # output channel, inputs and transformed kernels read once, no temporaries in memory).  It ranks before
    # every unfused tile.
    if C <= 4 and n2 * C <= vgpr_budget:
        nblocks = -(-tiles // 256)
        qread = nblocks * C * n2 * (256 + Kz)
        cands.append(((-(1 << 62), qread, 0, 0, Kz, 256),
                      dict(b=1, x=e * 256, y=e, z=Kz, alpha=C, threads=256, waves_m=1, waves_n=4,
                           path=PATH_FMA, wt_mode=1, lds_bytes_used=0, acc_regs_per_thread=n2 * C,
                           q_read_elems=qread, q_write_elems=N * K * P * Q)))
    # Fused blocks, any channel count: per channel a block reads the input windows of its tb sub-domains (a strip
    # of e tb + 2 by e + 2 pixels) and (e+2)^2 z transformed weights.  First where the time model prefers them.
    for fe, ftb, fz, falpha, fT, fwm, fwn, flds, facc in FUSED_BLOCKS:
        if fe != e or (lds_bytes and flds > lds_bytes) or (not auto_regs and facc > vgpr_budget):
            continue
        # byte offsets of a block's windows, counted from its first image, must stay below 2^30; a block of ftb
        # sub-domains touches at most ftb / (sub-domains per image) + 2 images
        per_image = (-(-P // e)) * (-(-Q // e))
        if (-(-ftb // per_image) + 2) * C * s["H"] * s["W"] * 4 >= 1 << 30:
            continue
        nblocks = (-(-tiles // ftb)) * (-(-K // fz))
        qread = nblocks * C * ((e * ftb + 2) * (e + 2) + n2 * fz)
        first = fused_faster(s, P, Q, e, ftb, fz, falpha)
        cands.append(((-(1 << 61) if first else 1, qread, 0, 0, fz, fT, falpha),
                      dict(b=1, x=e * ftb, y=e, z=fz, alpha=falpha, threads=fT, waves_m=fwm, waves_n=fwn,
                           path=PATH_FUSED, wt_mode=1, lds_bytes_used=flds, acc_regs_per_thread=facc,
                           q_read_elems=qread, q_write_elems=N * K * P * Q)))
    for tb in range(32, min(tb_top, 1024) + 1, 32):
        for z in divisors(Kz):
            if z % 32:
                continue
            if use_f3 and not (z * z <= sb_max and tb * tb <= sb_max):
                continue
            for _, T, _, wm, wn, acc in _wave_grids(z // 32, tb // 32, vgpr_budget, exact_only=True):   # tb is free: no idle blocks
                alpha = _pick_alpha(C, (16, 8, 4), 8 * (tb + z), lds_bytes if lds_bytes else _auto_lds_budget(T, acc), 2)
                if alpha is None:
                    continue
                ntb = -(-tiles // tb)
                nblocks = n2 * ntb * (Kz // z)
                qread = nblocks * C * (tb + z)
                cost = product_tile_cost(s, tb, z, alpha, T, wm, acc, nblocks, qread, n2 * Kz * ntb * tb)
                key = (0, cost, qread, abs(tb - z), -tb * z, z, T)
                cands.append((key, dict(b=1, x=e * tb, y=e, z=z, alpha=alpha, threads=T, waves_m=wm,
                                        waves_n=wn, path=PATH_MFMA, wt_mode=1,
                                        lds_bytes_used=(4 if alpha >= C else 8) * alpha * (tb + z), acc_regs_per_thread=acc,
                                        q_read_elems=qread, q_write_elems=N * K * P * Q)))
    return cands


def candidates(shape, lds_bytes=0, vgpr_budget=128, use_f3=True, auto_regs=True):
    """Every feasible tile with its ordering key (smaller is better); the MFMA path is preferred
    whenever it has a feasible tile.  Also what the exhaustive sweep enumerates (use_f3=False)."""
    s = shape
    P, Q = out_extent(s["H"], s["W"], s["R"], s["S"], s["stride"], s["pad"])
    if P < 1 or Q < 1:
        return []
    if s["algo"] == DIRECT:
        c = _direct_candidates(s, P, Q, lds_bytes, vgpr_budget, PATH_MFMA, use_f3)
        # the FMA path: when no matrix-core tile fits, and when none of them covers two blocks of 32 pixels --
        # very large kernels whose weight slab leaves the LDS room for a few pixels only.  FMA tiles carry no
        # modelled time: their keys start below zero and sort first.
        if max([t["b"] * t["x"] * t["y"] for _, t in c], default=0) < 64:
            c = c + _direct_candidates(s, P, Q, lds_bytes, vgpr_budget, PATH_FMA, use_f3)
        if pointwise_layer(s):
            c = c + _pointwise_candidates(s, P, Q, vgpr_budget, use_f3)
        if thin_direct_layer(s):
            c = c + _thin_direct_candidates(s, P, Q, vgpr_budget)
        return c
    e = WINO_E[s["algo"]]
    return _wino_candidates(s, P, Q, e, lds_bytes, vgpr_budget, use_f3, auto_regs)


def tune(shape, lds_bytes=0, vgpr_budget=128, auto_regs=True):
    """The tile the library's iolb_tune must return, or None when nothing fits.  Direct convolution ranks
    the whole domain by modelled time; Winograd looks inside the optimality box first."""
    c = candidates(shape, lds_bytes, vgpr_budget, shape["algo"] != DIRECT, auto_regs)
    if all(t["path"] == PATH_FUSED for _, t in c):
        c = candidates(shape, lds_bytes, vgpr_budget, False, auto_regs)   # tiny layers: drop the box
    if not c:
        return None
    return min(c, key=lambda kv: kv[0])[1]


def _volume_key(shape, t):
    """volume_order for a library tile (the thread count, then the matrix-core path, break the last ties); Winograd: the fused dataflow of
    Sec. 5.3 before the unfused tiles, whose temporaries make a round trip through memory that q_read does not
    count; unfused tiles by read volume, then |tb - z| (the optimality condition x y = r^2 z for sub-domain
    strips), then the fuller block."""
    if shape["algo"] == DIRECT and t["wt_mode"] == 2:
        return (t["q_read_elems"], abs(t["x"] - 9 * t["z"]), -t["x"] * t["z"], -t["x"], t["z"], 1, 1, 256, 0, 2)
    if shape["algo"] == DIRECT and t["path"] == PATH_POINT:
        # the same order on the image as one row of pixels: volume, distance from x y = R z, the fuller block ...
        return (t["q_read_elems"], abs(t["x"] - t["z"]), -t["x"] * t["z"], -t["x"], t["z"], 1, 1, 256, -PATH_POINT, t["alpha"])
    if shape["algo"] == DIRECT:
        P, Q = out_extent(shape["H"], shape["W"], shape["R"], shape["S"], shape["stride"], shape["pad"])
        return volume_order(shape["N"], shape["C"], P, Q, -(-shape["K"] // 32) * 32 if t["path"] == PATH_MFMA else shape["K"],
                            shape["R"], shape["S"], shape["stride"], t["b"], t["x"], t["y"], t["z"]) + (t["threads"], -t["path"])
    e = WINO_E[shape["algo"]]
    tb = t["x"] // e
    if t["path"] == PATH_FMA:
        return (-(1 << 62), 0, 0, 0, t["z"], 256, 0, 0)
    if t["path"] == PATH_FUSED:
        return (-(1 << 61), t["q_read_elems"], 0, 0, t["z"], t["threads"], 0, 0)
    return (0, t["q_read_elems"], abs(tb - t["z"]), -tb * t["z"], t["z"], t["threads"], 0, 0)


def bound_pick(shape, lds_bytes=0, vgpr_budget=128, auto_regs=True):
    """The tile the library's iolb_tune_bound must return: least reading volume (the paper's objective) among
    the tiles the kernels can run, inside the optimality box; the whole domain when the box is empty."""
    c = candidates(shape, lds_bytes, vgpr_budget, True, auto_regs) or candidates(shape, lds_bytes, vgpr_budget, False, auto_regs)
    if not c:
        return None
    return min((t for _, t in c), key=lambda t: _volume_key(shape, t))
