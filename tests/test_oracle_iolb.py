"""Pins for the bound/tuner oracle (oracle/iolb_oracle.py): hand-countable shapes, closed forms
and equality cases the paper states, and an independently written feasibility/optimality check
of the tile rule.  CPU only."""
from fractions import Fraction
from math import isclose, sqrt

import pytest

from oracle import iolb_oracle as o


def shape(N, C, H, W, K, R=3, S=3, stride=1, pad=1, algo=o.DIRECT):
    return dict(N=N, C=C, H=H, W=W, K=K, R=R, S=S, stride=stride, pad=pad, algo=algo)


def test_tree_vertex_counts():
    assert o.summation_tree(2) == (0, 1)             # Sec. 4.2: k inputs -> k-2 internal, 1 output
    assert o.summation_tree(9) == (7, 1)
    assert o.linear_combination_tree(4) == (6, 1)    # Sec. 4.3: 2k-2 internal, 1 output
    assert o.linear_combination_tree(16) == (30, 1)


def test_direct_vertex_count_hand_cases():
    assert o.V_DC(1, 1, 5, 7, 3, 1, 1) == 5 * 7 * 3              # 1x1x1 kernel: the outputs only... (2*1-1)
    assert o.V_DC(1, 1, 2, 2, 1, 2, 2) == 7 * 4                  # 4 products + 2 sums + 1 output each
    # count the DAG of a tiny layer vertex by vertex
    R, S, C, P, Q, K = 3, 2, 2, 2, 3, 2
    per_output = R * S * C + sum(o.summation_tree(R * S * C))
    assert o.V_DC(1, C, P, Q, K, R, S) == per_output * P * Q * K


def test_rho():
    assert o.rho(3, 3, 1) == 9
    assert o.rho(11, 11, 4) == Fraction(121, 16)
    assert o.rho(1, 1, 2) == Fraction(1, 4)


def test_direct_bound_worked_example():
    # rho = 9, S = 2, C = 2, 4x4 outputs, 2 kernels: every quantity is rational (2 rho S = 36)
    N, C, P, Q, K, R, S, st, Sf = 1, 2, 4, 4, 2, 3, 3, 1, 2
    V = o.V_DC(N, C, P, Q, K, R, S)
    assert V == 35 * 32 == 1120
    T4 = o.T_DC(2 * Sf, o.rho(R, S, st))
    assert T4 == 4 * 4 * 6 + 4 - 1 == 99
    general = o.general_lower_bound(V, T4, Sf)
    explicit = o.Qlow_DC_explicit(N, C, P, Q, K, R, S, st, Sf)
    assert general == explicit == Fraction(1120 * 2, 99) - 2          # both routes agree exactly
    assert isclose(float(general), 20.6262626, rel_tol=1e-8)
    lead = o.Qlow_DC_lead(N, C, P, Q, K, R, S, st, Sf)
    assert lead == Fraction(9 * 2 * 16 * 2, 4 * 6)


def test_direct_bound_general_equals_explicit_on_a_grid():
    for j in (1, 2, 3, 5):
        Sf = 2 * j * j                     # makes 2 rho S a perfect square for rho = 9
        for C in (1, 3, 8):
            V = o.V_DC(2, C, 6, 5, 4, 3, 3)
            g = o.general_lower_bound(V, o.T_DC(2 * Sf, Fraction(9)), Sf)
            assert g == o.Qlow_DC_explicit(2, C, 6, 5, 4, 3, 3, 1, Sf)


def test_dataflow_equality_cases():
    # direct: xy = rho z  (Sec. 5.2).  x = y = 12, z = 16, rho = 9:  z + xy/rho = 32 = 2 sqrt(xyz/rho)
    C, P, Q, K = 8, 24, 24, 32
    q = o.Qread_DC_paper(C, P, Q, K, 3, 3, 1, 12, 12, 16)
    assert q == o.Qread_DC_min(C, P, Q, K, 3, 3, 1, 12 * 12 * 16)
    assert q == Fraction(P * Q * K, 2304) * 9 * C * 32
    for x, y, z in ((12, 12, 8), (24, 12, 8), (6, 12, 32), (12, 6, 32), (12, 12, 32)):
        if x * y != 9 * z:
            assert o.Qread_DC_paper(C, P, Q, K, 3, 3, 1, x, y, z) > \
                   float(o.Qread_DC_min(C, P, Q, K, 3, 3, 1, x * y * z)) * (1 + 1e-12)
    # Winograd: xy = r^2 z (Sec. 5.3): (xy + 9z)/(xyz) = 1/8 = 2*3/sqrt(2304)
    qw = o.Qread_WA_paper(C, P, Q, K, 12, 12, 16)
    assert qw == o.Qread_WA_min(C, P, Q, K, 2304) == Fraction(P * Q * K * C, 8)


def test_dataflow_to_bound_ratios():
    # leading term of the dataflow volume over the printed bound at equal fast memory
    C, P, Q, K, Sf = 64, 56, 56, 64, 2 * 64 * 64
    lead_df = float(o.Q_DC_total(C, P, Q, K, 3, 3, 1, Sf)) - P * Q * K
    assert isclose(lead_df / float(o.Qlow_DC_lead(1, C, P, Q, K, 3, 3, 1, Sf)), 8 * sqrt(2), rel_tol=1e-12)
    for e in (2, 3, 4, 6):
        lead_w = float(o.Q_WA_total(C, P, Q, K, e, 4096)) - P * Q * K
        assert isclose(lead_w / float(o.Qlow_WA_lead(1, C, P, Q, K, e, 4096)), 2.0, rel_tol=1e-12)


def test_winograd_T_and_vertex_counts():
    assert o.T_WA(16, 2) == Fraction(2 * 64, 6) * 16 * 4 + Fraction(6 * 16, 6) * 16
    steps = o.V_WA_steps(C=10, e=2)
    n = 4
    assert steps["input_transform"] == 16 * sum(o.linear_combination_tree(16)) * 10
    assert steps["kernel_transform"] == 16 * sum(o.linear_combination_tree(9)) * 10
    assert steps["products"] == 160 and steps["channel_sums"] == 16 * sum(o.summation_tree(10))
    assert steps["output_transform"] == 4 * sum(o.linear_combination_tree(16))
    # the input transform carries the leading term 2 (e+r-1)^4 C per (tile, kernel)
    big = o.V_WA_steps(C=10 ** 6, e=4)
    lead = Fraction(2 * 6 ** 4 * 10 ** 6)
    assert 1 < Fraction(sum(big.values())) / lead < Fraction(3, 2)
    assert o.V_WA_lead(1, 3, 8, 8, 2, 4) == Fraction(2 * 64 * 2 * 3 * 6 ** 4, 16)


def test_winograd_bound_leading_term():
    v = o.Qlow_WA_lead(1, 64, 28, 28, 64, 2, 4096)
    assert v == Fraction(28 * 28 * 64 * 64 * 4 * 3, 2 * 64)


def test_compulsory():
    assert o.compulsory(2, 3, 5, 7, 4, 3, 3, 5, 7) == 2 * 3 * 35 + 4 * 3 * 9 + 2 * 4 * 35


# ---------------------------------------------------------------------------------------------
# tile rule
# ---------------------------------------------------------------------------------------------

def _check_feasible(s, cfg, lds_bytes, vgpr_budget):
    """Constraints re-stated from the documentation of the rule, written independently."""
    P, Q = o.out_extent(s["H"], s["W"], s["R"], s["S"], s["stride"], s["pad"])
    b, x, y, z, a, T = (cfg[k] for k in ("b", "x", "y", "z", "alpha", "threads"))
    if cfg["path"] == o.PATH_FMA and cfg["wt_mode"] == 2:
        # thin direct layers: 256 lanes, each tw neighbouring pixels of a row and every output channel
        assert (s["algo"], s["R"], s["S"], s["stride"]) == (o.DIRECT, 3, 3, 1) and s["C"] <= 4
        tw = 4 if Q % 4 == 0 else 1
        assert (b, x, y, z, a, T) == (1, 256 * tw, 1, s["K"], s["C"], 256) and cfg["lds_bytes_used"] == 0
        assert s["C"] * 3 * (tw + 2) <= vgpr_budget and cfg["acc_regs_per_thread"] == tw
        lanes = sum(len(range(0, Q, tw)) for _ in range(s["N"] * P))                # walked row by row
        assert cfg["q_read_elems"] == len(range(0, lanes, 256)) * s["C"] * (3 * (x + 2) + 9 * s["K"])
        assert cfg["q_write_elems"] == s["N"] * s["K"] * P * Q
        return
    if cfg["path"] == o.PATH_POINT:
        # 1 x 1 layers: four waves, each on x / 4 consecutive pixels of an image taken as one row, by z channels
        assert (s["algo"], s["R"], s["S"], s["pad"]) == (o.DIRECT, 1, 1, 0)
        assert (b, y, T, cfg["waves_m"], cfg["waves_n"]) == (1, 1, 256, 1, 4) and x % 128 == 0 and z % 32 == 0
        assert a in (16, 32) and (a == 16 or s["C"] % 32 == 0)
        assert cfg["acc_regs_per_thread"] == 16 * (x // 128) * (z // 32) <= vgpr_budget
        assert cfg["lds_bytes_used"] == 2 * 4 * a * z
        ranges = sum(len(range(0, P * Q, x // 4)) for _ in range(s["N"]))          # walked image by image
        groups = len(range(0, ranges, 4)) * len(range(0, s["K"], z))
        assert cfg["q_read_elems"] == groups * s["C"] * (x + z)
        assert cfg["q_write_elems"] == s["N"] * s["K"] * P * Q
        return
    if cfg["path"] == o.PATH_FUSED:
        # fused Winograd blocks (Sec. 5.3): every plane of a tb x z block in accumulator registers, one per kernel built
        e = o.WINO_E[s["algo"]]
        tb, planes = x // e, (e + 2) ** 2
        assert (e, tb, z, a, T) in ((2, 64, 64, 8, 1024), (4, 32, 64, 4, 768)) and (b, y) == (1, e)
        assert planes * tb * z == cfg["acc_regs_per_thread"] * T and cfg["acc_regs_per_thread"] <= vgpr_budget
        assert 2 * 4 * a * planes * (tb + z) <= cfg["lds_bytes_used"] <= (lds_bytes or o.LDS_CU)
        tiles = s["N"] * -(-P // e) * -(-Q // e)
        blocks = len(range(0, tiles, tb)) * len(range(0, s["K"], z))
        assert cfg["q_read_elems"] == blocks * s["C"] * ((e * tb + 2) * (e + 2) + planes * z)
        assert cfg["q_write_elems"] == s["N"] * s["K"] * P * Q
        return
    # matrix-core tiles cut K rounded up to whole 32-channel blocks
    Kz = -(-s["K"] // 32) * 32 if cfg["path"] == o.PATH_MFMA else s["K"]
    assert Kz % z == 0 and T in (64, 128, 256, 512, 1024)
    assert cfg["lds_bytes_used"] <= (lds_bytes or o.LDS_CU) and cfg["acc_regs_per_thread"] <= vgpr_budget
    if s["algo"] == o.DIRECT:
        # tile extents: factors of the output extent, or (matrix-core path) a balanced cut into up to 8 tiles
        ragged = cfg["path"] == o.PATH_MFMA
        assert s["N"] % b == 0
        assert Q % x == 0 or (ragged and any(x == -(-Q // k) for k in range(1, 9)))
        assert P % y == 0 or (ragged and any(y == -(-P // k) for k in range(1, 9)))
        halo = b * ((x - 1) * s["stride"] + s["S"]) * ((y - 1) * s["stride"] + s["R"])
        per_stage = halo + s["R"] * s["S"] * z
        blocks = (s["N"] // b) * -(-Q // x) * -(-P // y) * (Kz // z)
        assert cfg["q_read_elems"] == blocks * s["C"] * per_stage
        if cfg["path"] == o.PATH_MFMA:
            assert z % 32 == 0 and a % 4 == 0
            buffers = 1 if a >= s["C"] else 2                             # one stage only: one buffer
            assert cfg["lds_bytes_used"] == buffers * 4 * a * per_stage
            padded = -(-(b * x * y) // 32) * 32
            assert padded * z <= cfg["acc_regs_per_thread"] * T           # every output has a register
            assert cfg["acc_regs_per_thread"] * T < (padded + 32 * 8 * cfg["waves_n"]) * z
            assert T == 64 * cfg["waves_m"] * cfg["waves_n"]
        else:
            assert b * x * y <= 256 and cfg["lds_bytes_used"] == 4 * a * per_stage
    else:
        e = o.WINO_E[s["algo"]]
        assert b == 1 and y == e and x % (32 * e) == 0 and z % 32 == 0
        tb = x // e
        assert tb * z == cfg["acc_regs_per_thread"] * T
        assert cfg["lds_bytes_used"] == (4 if a >= s["C"] else 8) * a * (tb + z)     # one stage only: one buffer
    assert cfg["q_write_elems"] == s["N"] * s["K"] * P * Q


SHAPES = [shape(1, 16, 14, 14, 16), shape(8, 64, 28, 28, 64, algo=o.WINO_F2), shape(32, 64, 56, 56, 64),
          shape(64, 256, 14, 14, 256, algo=o.WINO_F4), shape(64, 3, 224, 224, 64),
          shape(64, 128, 112, 112, 128), shape(64, 512, 28, 28, 512), shape(16, 96, 27, 27, 256, 5, 5, 1, 2),
          shape(16, 3, 227, 227, 96, 11, 11, 4, 0), shape(4, 32, 32, 32, 64, algo=o.WINO_F4),
          shape(2, 8, 16, 16, 32, 1, 1, 1, 0), shape(3, 5, 9, 7, 6),
          shape(64, 256, 56, 56, 256, algo=o.WINO_F6), shape(8, 64, 28, 28, 64, algo=o.WINO_F3),
          shape(1, 16, 14, 14, 16, algo=o.WINO_F2), shape(4, 20, 13, 17, 48, algo=o.WINO_F4)]


@pytest.mark.parametrize("s", SHAPES)
@pytest.mark.parametrize("lds,vg", [(0, 128), (81920, 128), (32768, 64), (163840, 128)])
def test_tile_rule_returns_a_feasible_tile(s, lds, vg):
    cfg = o.tune(s, lds, vg)
    if cfg is None:
        assert not o.candidates(s, lds, vg, False)
        return
    _check_feasible(s, cfg, lds, vg)


def test_modelled_time_worked_example():
    """N=64, C=K=256, 56x56, 3x3; tile b=1, x=y=28, z=64, alpha=8, 8 waves as 2 x 4, 1 x 7 blocks per wave.
    By hand: halo 30*30 = 900 -> 15 chunks, 2 per wave -> 16 tile loads + ceil(8*9*16/512) = 3 weight loads;
    36 steps -> 36*7*64 = 16128 matrix-core cycles per wave and stage, own = 16128 + 36*8*32 + 300*19 = 31044;
    two waves per SIMD share 2 * (16128 + 36*8*8) = 36864 -> stage = max(36864, 31044) + 800 = 37664; 32 stages ->
    1205248 + 15000 + 200*112 = 1242648 per workgroup; 1024 workgroups = 4 rounds -> 4970592.  Memory: 1024*256*(900+576) elements
    read -> 386924 cycles, 51380224 written -> 137013: far below, so the time is the compute figure."""
    s = shape(64, 256, 56, 56, 256)
    q_read = 1024 * 256 * (900 + 576)
    assert o.mfma_tile_cost(s, 1, 28, 28, 64, 8, 512, 2, 112, 1024, q_read, 51380224) == 4970592
    # a tile whose rows are one pixel wide needs a load instruction per 64 elements as well, but moves
    # nine input elements per output: the memory term takes over
    wide = o.mfma_tile_cost(s, 64, 1, 1, 64, 8, 64, 2, 32, 64 * 56 * 56 * 4 // 64, 3136 * 4 * 256 * (576 + 576), 51380224)
    assert wide > 4970592


def test_modelled_time_properties():
    s = shape(64, 256, 56, 56, 256)
    base = dict(b=1, x=28, y=28, z=64, alpha=8, T=512, wm=2, acc=112)
    f = lambda nblocks, q: o.mfma_tile_cost(s, base["b"], base["x"], base["y"], base["z"], base["alpha"], base["T"],
                                            base["wm"], base["acc"], nblocks, q, 51380224)
    assert f(256, 10**6) == f(1, 10**6)                 # one round of the 256 compute units either way
    assert f(257, 10**6) == 2 * f(256, 10**6)           # one workgroup more: a second round
    # memory-bound: the volume decides; the 30-float rows of the 28-wide tile count as 128-byte requests
    rows, halo = 256 * 256 * 30, 256 * 256 * 900
    assert f(256, 10**12) == (rows * 128 + 4 * (10**12 - halo)) // 4000 + (4 * 51380224) // 1500


def test_optimality_box_prunes_and_holds_the_bound_pick():
    """Table 1: the box z <= sqrt(S_b/rho), b x y <= sqrt(S_b rho) prunes the domain, and the bound-only pick
    (least reading volume) lies inside it.  This build's heuristic pick need not: it ranks the whole domain."""
    sb = o.T_MAX * 128
    for s in (shape(64, 256, 56, 56, 256), shape(32, 64, 56, 56, 64), shape(64, 128, 112, 112, 128), shape(16, 96, 27, 27, 256, 5, 5, 1, 2)):
        inside = o.candidates(s, use_f3=True)
        everything = o.candidates(s, use_f3=False)
        assert 0 < len(inside) < len(everything)
        RS, st2 = s["R"] * s["S"], s["stride"] ** 2
        for _, c in inside:
            assert c["z"] ** 2 * RS <= sb * st2 and (c["b"] * c["x"] * c["y"]) ** 2 * st2 <= sb * RS
        pick = o.bound_pick(s)
        assert pick in [c for _, c in inside]
        assert pick["q_read_elems"] == min(c["q_read_elems"] for _, c in inside)


# ---------------------------------------------------------------------------------------------
# the paper's rule (Table 1 domain, reading volume of Sec. 5.2): pins that do not come from the oracle itself
# ---------------------------------------------------------------------------------------------

def _count_reads_by_walking_the_blocks(N, C, P, Q, K, R, S, stride, b, x, y, z):
    """The dataflow of Sec. 5.2 walked block by block: per block and input channel, the pixels of the input
    tile under the block (counted one by one from the first and last window of each axis) and the weights of
    the block's kernels."""
    total = 0
    for n0 in range(0, N, b):
        for q0 in range(0, Q, x):
            for p0 in range(0, P, y):
                for k0 in range(0, K, z):
                    cols = len(range(q0 * stride, (q0 + x - 1) * stride + S))     # first pixel of the first window .. last of the last
                    rows = len(range(p0 * stride, (p0 + y - 1) * stride + R))
                    total += C * (b * rows * cols + R * S * z)
    return total


def test_reading_volume_equals_a_walk_over_the_blocks():
    import random
    rnd = random.Random(11)
    for _ in range(60):
        N, C, P, Q, K = rnd.choice([1, 2, 4]), rnd.randint(1, 5), rnd.choice([4, 6, 8, 12]), rnd.choice([4, 6, 9, 12]), rnd.choice([4, 8, 12])
        R, S, st = rnd.choice([1, 2, 3]), rnd.choice([1, 3, 5]), rnd.choice([1, 2])
        b, x, y, z = (rnd.choice(o.divisors(v)) for v in (N, Q, P, K))
        assert o.Qread_exact(N, C, P, Q, K, R, S, st, b, x, y, z) == \
               _count_reads_by_walking_the_blocks(N, C, P, Q, K, R, S, st, b, x, y, z)


def test_reading_volume_approaches_the_papers_expression():
    """With x' ~ mu x, as Sec. 5.2 takes it, the exact volume becomes (H W C_out / xyz) W_ker H_ker C_in (z + xy/rho)
    for stride = kernel extent (no overlap between windows: the approximation is then exact)."""
    C, P, Q, K = 3, 12, 12, 8
    for x, y, z in ((2, 3, 4), (6, 4, 8), (12, 12, 1)):
        assert o.Qread_exact(1, C, P, Q, K, 2, 2, 2, 1, x, y, z) == o.Qread_DC_paper(C, P, Q, K, 2, 2, 2, x, y, z)


def test_bound_rule_worked_example():
    """S_b = 2304, rho = 9, 24 x 24 outputs, 32 kernels: the box is z <= 16, x y <= 144, and x y = rho z is met
    by x y = 144, z = 16 -- reached by (12, 12), (6, 24), (24, 6).  With the true input tile, (x + 2)(y + 2), the
    square block reads least: 8 blocks of (14 * 14 + 9 * 16) elements per channel."""
    N, C, P, Q, K = 1, 5, 24, 24, 32
    dom = o.paper_domain(N, P, Q, K, 3, 3, 1, 2304)
    assert max(z for _, _, _, z in dom) == 16 and max(b * x * y for b, x, y, _ in dom) == 144
    assert {(1, 12, 12, 16), (1, 6, 24, 16), (1, 24, 6, 16)} <= set(dom)
    pick = o.tune_by_volume(N, C, P, Q, K, 3, 3, 1, 2304)
    assert pick == (1, 12, 12, 16)
    assert o.Qread_exact(N, C, P, Q, K, 3, 3, 1, *pick) == 8 * C * (196 + 144)
    # the three tiles on the optimality curve tie in the paper's approximate expression
    vols = {o.Qread_DC_paper(C, P, Q, K, 3, 3, 1, x, y, 16) for x, y in ((12, 12), (6, 24), (24, 6))}
    assert len(vols) == 1


def test_bound_rule_is_the_argmin_over_an_independent_enumeration():
    """Brute force on small layers: no tile of the Table 1 domain, listed here with itertools and its volume
    counted by walking the blocks, reads less than the rule's pick; ties are broken towards x y = rho z."""
    import itertools
    import random
    rnd = random.Random(3)
    checked = 0
    for _ in range(200):
        N, C = rnd.choice([1, 2, 4]), rnd.randint(1, 4)
        P, Q, K = rnd.choice([4, 6, 8, 12]), rnd.choice([4, 6, 8, 12]), rnd.choice([4, 8, 16])
        R = S = rnd.choice([1, 3])
        st = rnd.choice([1, 2])
        Sb = rnd.choice([64, 256, 576])
        pick = o.tune_by_volume(N, C, P, Q, K, R, S, st, Sb)
        listed = [(b, x, y, z) for b, x, y, z in itertools.product(range(1, N + 1), range(1, Q + 1), range(1, P + 1), range(1, K + 1))
                  if N % b == 0 and Q % x == 0 and P % y == 0 and K % z == 0 and b * x * y * z <= Sb
                  and (z * z * R * S) <= Sb * st * st and (b * x * y * st) ** 2 <= Sb * R * S]
        if not listed:
            assert pick is None
            continue
        vol = {t: _count_reads_by_walking_the_blocks(N, C, P, Q, K, R, S, st, *t) for t in listed}
        least = min(vol.values())
        assert vol[pick] == least
        ties = [t for t in listed if vol[t] == least]
        dist = lambda t: abs(t[0] * t[1] * t[2] * st * st - R * S * t[3])
        assert dist(pick) == min(dist(t) for t in ties)
        checked += 1
    assert checked > 150


def test_more_fast_memory_never_reads_more():
    """The domain only grows with S_b (and with the LDS budget): the least reading volume cannot rise."""
    vols = [o.Qread_exact(4, 16, 28, 28, 64, 3, 3, 1, *o.tune_by_volume(4, 16, 28, 28, 64, 3, 3, 1, Sb))
            for Sb in (64, 256, 1024, 4096, 16384)]
    assert vols == sorted(vols, reverse=True) and vols[0] > vols[-1]
    s = shape(64, 256, 56, 56, 256)
    reads = [o.bound_pick(s, lds, 128)["q_read_elems"] for lds in (24576, 40960, 81920, 163840)]
    assert reads == sorted(reads, reverse=True) and reads[0] > reads[-1]


def test_bound_pick_runs_the_papers_winograd_dataflow():
    """Sec. 5.3 keeps every temporary on chip: where a fused block exists the bound-only pick is one; without one
    (F(3x3), F(6x6)) it is the unfused tile of least reading volume."""
    assert o.bound_pick(shape(64, 128, 112, 112, 128, algo=o.WINO_F4))["path"] == o.PATH_FUSED
    assert o.bound_pick(shape(64, 3, 224, 224, 64, algo=o.WINO_F2))["path"] == o.PATH_FMA          # thin: one-kernel FMA path
    s = shape(8, 64, 28, 28, 64, algo=o.WINO_F3)
    pick = o.bound_pick(s)
    assert pick["path"] == o.PATH_MFMA
    assert pick["q_read_elems"] == min(c["q_read_elems"] for _, c in o.candidates(s, use_f3=True))


def test_continuous_optimum_is_on_the_optimality_curve():
    """With the paper's approximate halo (x' ~ x) the read volume over tiles of equal volume is
    smallest where xy = rho z: check on S_b = 2304, rho = 9 that (xy, z) = (144, 16) wins."""
    C, P, Q, K = 4, 24, 24, 32
    best = None
    for x in o.divisors(Q):
        for y in o.divisors(P):
            for z in o.divisors(K):
                if x * y * z == 2304:
                    v = o.Qread_DC_paper(C, P, Q, K, 3, 3, 1, x, y, z)
                    if best is None or v < best[0]:
                        best = (v, {(x * y, z)})
                    elif v == best[0]:
                        best[1].add((x * y, z))
    assert best[1] == {(144, 16)}


def test_more_lds_never_costs_more():
    """Heuristic order: a larger LDS budget only adds feasible tiles and deeper stages, so the modelled time of the
    pick cannot rise (a property of this build's model, no pin of the paper's rule)."""
    s = shape(64, 256, 56, 56, 256)
    costs = [min(k[0] for k, _ in o.candidates(s, lds, 128, use_f3=False)) for lds in (24576, 40960, 81920, 163840)]
    assert costs == sorted(costs, reverse=True) and costs[0] > costs[-1]


def test_no_tile_when_nothing_fits():
    assert o.tune(shape(1, 16, 14, 14, 16), lds_bytes=16, vgpr_budget=128) is None


def test_bounds_report():
    s = shape(32, 64, 56, 56, 64)
    r = o.bounds(s, 20480)
    assert r["compulsory_elems"] == 32 * 64 * 3136 + 64 * 64 * 9 + 32 * 64 * 3136
    assert r["vertices"] == (2 * 9 * 64 - 1) * 56 * 56 * 64 * 32
    assert isclose(r["q_lower_lead"], 9 * 64 * 3136 * 64 * 32 / (4 * sqrt(2 * 9 * 20480)), rel_tol=1e-12)


def test_thin_winograd_layers_get_the_fused_candidate_first():
    """C <= 4 and C (e+2)^2 <= register budget: the one-kernel dataflow of Sec. 5.3 is a candidate, ranks
    first, covers every output channel with 256 sub-domains per workgroup and uses no LDS; otherwise every
    candidate is a matrix-core tile (unfused, or a fused block)."""
    for algo, e in o.WINO_E.items():
        n2 = (e + 2) ** 2
        for C in range(1, 7):
            for budget in (128, 64):
                s = dict(N=2, C=C, H=20, W=24, K=40, R=3, S=3, stride=1, pad=1, algo=algo)
                cands = o.candidates(s, 0, budget, use_f3=False)
                fused = [c for _, c in cands if c["path"] == o.PATH_FMA]
                if C <= 4 and n2 * C <= budget:
                    assert len(fused) == 1
                    f = fused[0]
                    assert o.tune(s, 0, budget) == f
                    tiles = 2 * -(-20 // e) * -(-24 // e)
                    assert (f["x"], f["y"], f["z"], f["alpha"], f["threads"]) == (256 * e, e, 64, C, 256)
                    assert f["lds_bytes_used"] == 0 and f["acc_regs_per_thread"] == n2 * C
                    assert f["q_read_elems"] == -(-tiles // 256) * C * n2 * (256 + 64)
                    assert f["q_write_elems"] == 2 * 40 * 20 * 24
                else:
                    assert not fused
                    assert o.tune(s, 0, budget)["path"] in (o.PATH_MFMA, o.PATH_FUSED)


def test_single_stage_tiles_count_one_buffer_and_large_kernels_fall_back_to_fma():
    """A layer whose channels fit one stage (C <= alpha) keeps a single LDS buffer, which admits tiles twice
    as large (7x7 stride-2 first layer: more than 80 KB in one buffer, eight waves).  An 11x11 stride-4 first
    layer, whose weight slab leaves room for 25 pixels only, is handed to the FMA path."""
    s = shape(64, 3, 224, 224, 64, 7, 7, 2, 3)
    t = o.tune(s)
    halo = t["b"] * ((t["x"] - 1) * 2 + 7) * ((t["y"] - 1) * 2 + 7)
    assert t["path"] == o.PATH_MFMA and t["alpha"] == 4 and t["threads"] == 512
    assert t["lds_bytes_used"] == 4 * 4 * (halo + 49 * t["z"]) and 81920 < t["lds_bytes_used"] <= o.LDS_CU
    a = o.tune(shape(16, 3, 227, 227, 96, 11, 11, 4, 0))
    assert a["path"] == o.PATH_FMA
    # with more channels than a stage holds the same 7x7 layer needs both buffers again
    t2 = o.tune(shape(64, 8, 224, 224, 64, 7, 7, 2, 3))
    halo2 = t2["b"] * ((t2["x"] - 1) * 2 + 7) * ((t2["y"] - 1) * 2 + 7)
    assert t2["alpha"] < 8 or t2["lds_bytes_used"] == 4 * t2["alpha"] * (halo2 + 49 * t2["z"])
    if t2["alpha"] < 8:
        assert t2["lds_bytes_used"] == 8 * t2["alpha"] * (halo2 + 49 * t2["z"])


def test_tile_extents_are_factors_plus_balanced_cuts():
    assert o.tile_extents(35, o.PATH_MFMA) == [1, 5, 6, 7, 9, 12, 18, 35]       # factors 1, 5, 7, 35; ceil(35/k), k <= 8
    assert o.tile_extents(35, o.PATH_FMA) == [1, 5, 7, 35]
    assert o.tile_extents(56, o.PATH_MFMA) == [1, 2, 4, 7, 8, 14, 28, 56]          # eight factors: no cuts needed
    assert o.tile_extents(28, o.PATH_MFMA) == [1, 2, 4, 5, 6, 7, 10, 14, 28]        # six factors: cuts admitted
    # a cut into k tiles covers the extent with the last tile hanging over by less than k pixels
    for n in (13, 27, 55, 73, 147, 149):
        for x in o.tile_extents(n, o.PATH_MFMA):
            k = -(-n // x)
            assert (k - 1) * x < n <= k * x
