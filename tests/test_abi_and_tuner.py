"""CPU-side checks of the C-ABI library: it loads, exports what the header declares, and its
tuner / bound figures agree with the oracle (bit-exactly for every integer).  No GPU needed."""
import os
import re

import pytest

from oracle import iolb_oracle as o
from paper_2012_15667_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "iolbconv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b((?:conv|iolb)_[a-z_0-9]+)\s*\(", text))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    declared = _declared_symbols()
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_strerror():
    L = B.lib()
    assert L.iolb_strerror(0) == b"success"
    assert b"tile" in L.iolb_strerror(-3)


def _shape(N, C, H, W, K, R=3, S=3, stride=1, pad=1, algo=0):
    return dict(N=N, C=C, H=H, W=W, K=K, R=R, S=S, stride=stride, pad=pad, algo=algo)


SHAPES = [
    _shape(1, 16, 14, 14, 16), _shape(8, 64, 28, 28, 64, algo=1), _shape(32, 64, 56, 56, 64),
    _shape(64, 256, 14, 14, 256, algo=2), _shape(64, 256, 14, 14, 256), _shape(64, 3, 224, 224, 64),
    _shape(64, 128, 112, 112, 128), _shape(64, 256, 56, 56, 256), _shape(64, 512, 28, 28, 512),
    _shape(64, 3, 224, 224, 64, algo=1), _shape(64, 128, 112, 112, 128, algo=2), _shape(64, 512, 28, 28, 512, algo=1),
    _shape(16, 3, 227, 227, 96, 11, 11, 4, 0), _shape(16, 96, 27, 27, 256, 5, 5, 1, 2),
    _shape(16, 256, 13, 13, 384), _shape(16, 384, 13, 13, 256, algo=2), _shape(16, 256, 13, 13, 384, algo=1),
    _shape(2, 8, 16, 16, 32, 1, 1, 1, 0), _shape(3, 5, 9, 7, 6), _shape(4, 32, 32, 32, 64), _shape(4, 32, 32, 32, 64, algo=2),
    _shape(2, 6, 20, 12, 96, 3, 3, 2, 1), _shape(1, 1, 1, 1, 1, 1, 1, 1, 0), _shape(5, 7, 11, 13, 17, 2, 3, 1, 1),
    _shape(64, 256, 56, 56, 256, algo=4), _shape(64, 128, 112, 112, 128, algo=3), _shape(8, 64, 28, 28, 64, algo=3),
    _shape(4, 20, 13, 17, 96, algo=4), _shape(1, 16, 14, 14, 16, algo=1), _shape(4, 20, 13, 17, 48, algo=2),
    _shape(2, 16, 13, 13, 80), _shape(2, 64, 7, 7, 1000, 1, 1, 1, 0),
    # thin Winograd layers: fused one-kernel candidate when C <= 4 and C (m+2)^2 fits the register budget
    _shape(64, 3, 224, 224, 64, algo=2), _shape(2, 4, 37, 41, 33, algo=1), _shape(2, 4, 14, 14, 32, algo=2),
    _shape(2, 2, 14, 14, 32, algo=4), _shape(2, 3, 14, 14, 32, algo=4), _shape(1, 1, 9, 9, 5, algo=3),
    _shape(64, 192, 35, 35, 64, 1, 1, 1, 0), _shape(64, 1280, 8, 8, 384, 1, 1, 1, 0), _shape(8, 20, 17, 18, 70, 1, 1, 1, 0),
]
BUDGETS = [(0, 0), (32768, 64), (163840, 128), (8192, 32)]


@pytest.mark.parametrize("s", SHAPES)
@pytest.mark.parametrize("lds,vg", BUDGETS)
def test_tuner_bit_exact_against_oracle(s, lds, vg):
    want = o.tune(s, lds, vg or 128, auto_regs=(vg == 0))
    sh = B.make_shape(**s)
    if want is None:
        with pytest.raises(B.IolbError) as e:
            B.iolb_tune(sh, lds, vg)
        assert e.value.code == -3
    else:
        assert B.iolb_tune(sh, lds, vg) == want


@pytest.mark.parametrize("s", SHAPES)
@pytest.mark.parametrize("lds,vg", BUDGETS)
def test_bound_only_pick_bit_exact_against_oracle(s, lds, vg):
    """iolb_tune_bound (least reading volume inside the optimality box) against the oracle's bound_pick."""
    want = o.bound_pick(s, lds, vg or 128, auto_regs=(vg == 0))
    sh = B.make_shape(**s)
    if want is None:
        with pytest.raises(B.IolbError) as e:
            B.iolb_tune_bound(sh, lds, vg)
        assert e.value.code == -3
    else:
        assert B.iolb_tune_bound(sh, lds, vg) == want


def test_bound_only_pick_minimises_the_reading_volume_of_the_enumerated_box():
    """Against the library's own enumeration: no direct-convolution tile inside the box reads less."""
    for s in SHAPES:
        if s["algo"] != 0:
            continue
        sh = B.make_shape(**s)
        inside = B.iolb_enumerate(sh, 0, 0, True) or B.iolb_enumerate(sh, 0, 0, False)
        if not inside:
            continue
        pick = B.iolb_tune_bound(sh)
        assert pick in inside
        assert pick["q_read_elems"] == min(t["q_read_elems"] for t in inside)


@pytest.mark.parametrize("s", SHAPES[:9] + SHAPES[12:14] + SHAPES[18:])
@pytest.mark.parametrize("box", [True, False])
def test_enumeration_bit_exact_and_in_order(s, box):
    want = [c for _, c in sorted(o.candidates(s, use_f3=box), key=lambda kc: kc[0])]
    got = B.iolb_enumerate(B.make_shape(**s), 0, 0, box)
    assert got == want


def test_random_small_shapes_bit_exact():
    import random
    rnd = random.Random(5)
    for _ in range(150):
        R = rnd.choice([1, 2, 3, 5])
        s = _shape(rnd.choice([1, 2, 4, 6, 8]), rnd.randint(1, 40), rnd.randint(5, 40), rnd.randint(5, 40),
                   rnd.choice([8, 16, 24, 32, 64, 96]), R, rnd.choice([1, 2, 3]), rnd.choice([1, 2]), rnd.choice([0, 1, 2]))
        if s["H"] + 2 * s["pad"] < s["R"] or s["W"] + 2 * s["pad"] < s["S"]:
            continue
        want = o.tune(s)
        sh = B.make_shape(**s)
        if want is None:
            with pytest.raises(B.IolbError):
                B.iolb_tune(sh)
        else:
            assert B.iolb_tune(sh) == want, s
            assert B.iolb_tune_bound(sh) == o.bound_pick(s), s


@pytest.mark.parametrize("s", SHAPES[:12] + SHAPES[24:])
@pytest.mark.parametrize("Sf", [2, 20480, 40960, 44_000_000])
def test_bounds_match_oracle(s, Sf):
    got = B.iolb_bounds(B.make_shape(**s), Sf)
    want = o.bounds(s, Sf)
    for k in ("P", "Q", "vertices", "compulsory_elems", "q_write_elems"):
        assert got[k] == want[k], k
    for k in ("t_bound_2s", "q_lower_lead", "q_lower_explicit", "q_dataflow"):
        assert got[k] == pytest.approx(want[k], rel=1e-12, abs=1e-9), k


def test_invalid_arguments_are_rejected_without_a_gpu():
    with pytest.raises(B.IolbError) as e:
        B.iolb_tune(B.make_shape(0, 1, 4, 4, 1))
    assert e.value.code == -1
    with pytest.raises(B.IolbError) as e:
        B.iolb_tune(B.make_shape(1, 1, 4, 4, 32, 5, 5, 1, 1, algo=1))
    assert e.value.code == -2
    with pytest.raises(B.IolbError) as e:
        B.iolb_tune(B.make_shape(1, 1, 2, 2, 1, 5, 5, 1, 0))
    assert e.value.code == -1
    assert B.winograd_workspace_bytes(1, 8, 8, 8, 32, 5) == 0
    assert B.winograd_workspace_bytes(1, 8, 8, 8, 32, 3) > 0
    assert B.winograd_workspace_bytes(1, 8, 8, 8, 32, 4) > 0
    # the padded entry points check their arguments before any GPU call (the pointers are never followed)
    import ctypes
    L = B.lib()
    fake = [ctypes.c_void_p(4096)] * 3
    assert L.conv_direct_pad2(None, None, None, 1, 4, 8, 8, 32, 3, 3, 1, 1, 1) == -1
    assert L.conv_direct_pad2(*fake, 1, 4, 8, 8, 32, 3, 3, 1, -1, 0) == -1
    assert L.conv_direct_pad2(*fake, 1, 4, 8, 4, 32, 1, 7, 1, 0, 1) == -1          # W + 2 pad_w < S
    assert L.conv_direct_pad2(*fake, 1, 4, 8, 8, 32, 3, 3, 0, 1, 1) == -1          # stride 0
    assert L.conv_winograd_pad(None, None, None, 1, 4, 8, 8, 32, 4, 1) == -1
    assert L.conv_winograd_pad(*fake, 1, 4, 8, 8, 32, 5, 1) == -2                   # m = 5
    assert L.conv_winograd_pad(*fake, 1, 4, 8, 8, 32, 4, -1) == -1
    assert L.conv_winograd_pad(*fake, 1, 4, 2, 2, 32, 4, 0) == -1                   # H + 2 pad < 3


@pytest.mark.parametrize("m", [2, 3, 4, 6])
def test_library_winograd_matrices_satisfy_the_defining_identity(m):
    """The constants compiled into the Winograd kernels: for output i, tap j and input k,
    sum_xi A[i][xi] L[xi][j] B[xi][k] = [k == i + j]  (1-D F(m, 3); the 2-D transforms nest it).
    Checked on the library's own floats, no oracle involved."""
    from fractions import Fraction
    A, Lm, Bm = B.iolb_winograd_matrices(m)
    n = m + 2
    assert len(A) == m and len(Lm) == n and len(Bm) == n
    for i in range(m):
        for j in range(3):
            for k in range(n):
                s = sum(Fraction(A[i][xi]) * Fraction(Lm[xi][j]) * Fraction(Bm[xi][k]) for xi in range(n))
                scale = sum(abs(Fraction(A[i][xi]) * Fraction(Lm[xi][j]) * Fraction(Bm[xi][k])) for xi in range(n))
                assert abs(s - (1 if k == i + j else 0)) <= Fraction(1, 10**6) * max(1, scale), (i, j, k)
    with pytest.raises(B.IolbError) as e:
        B.iolb_winograd_matrices(5)
    assert e.value.code == -2


def test_maximum_tensor_sizes():
    """Tensors hold at most 2^31 - 1 elements: one element more is rejected before anything is tuned."""
    ok = B.make_shape(32767, 64, 32, 32, 64)            # x: 2^31 - 65536 elements
    cfg = B.iolb_tune(ok)
    assert 32767 % cfg["b"] == 0 and cfg["q_write_elems"] == 32767 * 64 * 32 * 32
    for bad in (B.make_shape(32768, 64, 32, 32, 64),    # x: exactly 2^31
                B.make_shape(1, 1, 4, 4, 2 ** 27, 4, 4, 1, 0),   # w: 2^31
                B.make_shape(32768, 1, 32, 32, 64)):    # y: 2^31
        with pytest.raises(B.IolbError) as e:
            B.iolb_tune(bad)
        assert e.value.code == -1


def test_fused_blocks_leave_the_domain_where_their_offsets_would_not_fit():
    """The fused Winograd kernels address a block's input windows with byte offsets below 2^30 from the block's first
    image (a block touches at most tb / (sub-domains per image) + 2 images): a layer whose images are larger than
    that gets no fused block, in either implementation, and still gets a tile."""
    small = _shape(2, 64, 512, 512, 64, 3, 3, 1, 1, algo=o.WINO_F4)       # 3 images of 64 MiB
    large = _shape(2, 96, 1024, 1024, 64, 3, 3, 1, 1, algo=o.WINO_F4)     # 3 images of 384 MiB
    for s, has in ((small, True), (large, False)):
        got = B.iolb_enumerate(B.make_shape(**s), 0, 0, False)
        want = [c for _, c in sorted(o.candidates(s, use_f3=False), key=lambda kc: kc[0])]
        assert got == want
        assert any(t["path"] == o.PATH_FUSED for t in got) == has
        assert B.iolb_tune(B.make_shape(**s)) == o.tune(s)

