"""Pins for the convolution oracle (oracle/conv_ref.c): hand-computed cases, exact brute force,
invariants, and special cases that reduce to library routines.  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle.conv_oracle import conv_ref, conv_ref_cwh, conv_ref_hwc, conv_ref_points, out_extent
from paper_2012_15667_amd.inputs import make_inputs, sample_output_indices

GOLD = os.path.join(os.path.dirname(__file__), "golden", "conv_hand_cases.txt")


def _gold(case):
    out = []
    for line in open(GOLD):
        t = line.split()
        if t and t[0] == case:
            out.append((int(t[1]), int(t[2]), float(t[3])))
    return out


def test_hand_case_all_ones_kernel():
    x = np.arange(1, 10, dtype=np.float32).reshape(1, 1, 3, 3)
    w = np.ones((1, 1, 3, 3), dtype=np.float32)
    y = conv_ref(x, w, 1, 1)
    assert y.shape == (1, 1, 3, 3)
    for p, q, v in _gold("A"):
        assert y[0, 0, p, q] == v


def test_hand_case_stride2():
    x = np.arange(1, 17, dtype=np.float32).reshape(1, 1, 4, 4)
    w = np.array([[1, 2], [3, 4]], dtype=np.float32).reshape(1, 1, 2, 2)
    y = conv_ref(x, w, 2, 0)
    assert y.shape == (1, 1, 2, 2)
    for p, q, v in _gold("B"):
        assert y[0, 0, p, q] == v


def test_hand_case_orientation():
    x = np.arange(1, 10, dtype=np.float32).reshape(1, 1, 3, 3)
    w = np.zeros((1, 1, 3, 3), dtype=np.float32)
    w[0, 0, 0, 0] = 1
    y = conv_ref(x, w, 1, 1)
    for p, q, v in _gold("C"):
        assert y[0, 0, p, q] == v


def _brute_fraction(x, w, stride, pad):
    """Independent second expression of the definition, in exact rationals, gathering the
    window first and then summing products (different loop structure from the C file)."""
    N, C, H, W = x.shape
    K, _, R, S = w.shape
    P = (H + 2 * pad - R) // stride + 1
    Q = (W + 2 * pad - S) // stride + 1
    xp = [[[[Fraction(0)] * (W + 2 * pad) for _ in range(H + 2 * pad)] for _ in range(C)] for _ in range(N)]
    for n in range(N):
        for c in range(C):
            for h in range(H):
                for ww in range(W):
                    xp[n][c][h + pad][ww + pad] = Fraction(float(x[n, c, h, ww]))
    y = np.empty((N, K, P, Q), dtype=object)
    for n in range(N):
        for k in range(K):
            for p in range(P):
                for q in range(Q):
                    window = [(xp[n][c][p * stride + r][q * stride + s], Fraction(float(w[k, c, r, s])))
                              for s in range(S) for r in range(R) for c in range(C)]
                    y[n, k, p, q] = sum(a * b for a, b in window)
    return y


@pytest.mark.parametrize("N,C,H,W,K,R,S,stride,pad", [
    (2, 3, 5, 6, 2, 3, 3, 1, 1),
    (1, 2, 7, 5, 3, 3, 2, 2, 0),
    (1, 1, 9, 9, 2, 5, 5, 1, 2),
    (2, 2, 11, 11, 2, 4, 4, 3, 1),
    (1, 3, 6, 4, 2, 1, 1, 1, 0),
    (1, 2, 8, 8, 1, 3, 3, 2, 2),
])
def test_brute_force_exact_small_integers(N, C, H, W, K, R, S, stride, pad):
    rng = np.random.default_rng(7)
    x = rng.integers(-4, 5, size=(N, C, H, W)).astype(np.float32)
    w = rng.integers(-3, 4, size=(K, C, R, S)).astype(np.float32)
    y = conv_ref(x, w, stride, pad)
    ref = _brute_fraction(x, w, stride, pad)
    assert y.shape == ref.shape
    for got, want in zip(y.ravel(), ref.ravel()):
        assert Fraction(float(got)) == want          # small integers: fp64 is exact


@pytest.mark.parametrize("N,C,H,W,K,R,S,stride,pad", [(2, 3, 5, 6, 4, 3, 3, 1, 1), (1, 2, 7, 5, 3, 3, 2, 2, 0)])
def test_hwc_layout_brute_force_in_its_own_index_order(N, C, H, W, K, R, S, stride, pad):
    """Channels-innermost tensors: y[n,p,q,k] = sum x[n, p*stride+r-pad, q*stride+s-pad, c] w[k,c,r,s],
    summed here directly on the HWC arrays (small integers, exact)."""
    rng = np.random.default_rng(11)
    x = rng.integers(-4, 5, size=(N, H, W, C)).astype(np.float32)
    w = rng.integers(-3, 4, size=(K, C, R, S)).astype(np.float32)
    y = conv_ref_hwc(x, w, stride, pad)
    P, Q = out_extent(H, W, R, S, stride, pad)
    assert y.shape == (N, P, Q, K)
    for n in range(N):
        for p in range(P):
            for q in range(Q):
                for k in range(K):
                    acc = 0
                    for r in range(R):
                        for s in range(S):
                            h, ww = p * stride + r - pad, q * stride + s - pad
                            if 0 <= h < H and 0 <= ww < W:
                                for c in range(C):
                                    acc += int(x[n, h, ww, c]) * int(w[k, c, r, s])
                    assert y[n, p, q, k] == acc


def test_cwh_layout_brute_force_in_its_own_index_order():
    """W before H: y[n,k,q,p] = sum x[n, c, q*stride+s-pad, p*stride+r-pad] w[k,c,r,s], summed on the CWH arrays."""
    N, C, H, W, K, R, S, stride, pad = 2, 2, 5, 7, 3, 2, 3, 1, 1
    rng = np.random.default_rng(12)
    x = rng.integers(-4, 5, size=(N, C, W, H)).astype(np.float32)
    w = rng.integers(-3, 4, size=(K, C, R, S)).astype(np.float32)
    y = conv_ref_cwh(x, w, stride, pad)
    P, Q = out_extent(H, W, R, S, stride, pad)
    assert y.shape == (N, K, Q, P)
    for n in range(N):
        for k in range(K):
            for q in range(Q):
                for p in range(P):
                    acc = 0
                    for c in range(C):
                        for r in range(R):
                            for s in range(S):
                                h, ww = p * stride + r - pad, q * stride + s - pad
                                if 0 <= h < H and 0 <= ww < W:
                                    acc += int(x[n, c, ww, h]) * int(w[k, c, r, s])
                    assert y[n, k, q, p] == acc


def test_delta_kernel_reproduces_input_bitwise():
    x, _ = make_inputs(2, 5, 9, 7, 5, 3, 3, seed=3)
    w = np.zeros((5, 5, 3, 3), dtype=np.float32)
    for k in range(5):
        w[k, k, 1, 1] = 1.0
    y = conv_ref(x, w, 1, 1)
    assert np.array_equal(y, x.astype(np.float64))


def test_shifted_delta_shifts_and_zero_border():
    x, _ = make_inputs(1, 2, 6, 8, 2, 3, 3, seed=4)
    w = np.zeros((2, 2, 3, 3), dtype=np.float32)
    w[0, 0, 0, 0] = 1.0          # top-left tap
    w[1, 1, 2, 1] = 1.0          # bottom-centre tap
    y = conv_ref(x, w, 1, 1)
    want0 = np.zeros((6, 8)); want0[1:, 1:] = x[0, 0, :-1, :-1]
    want1 = np.zeros((6, 8)); want1[:-1, :] = x[0, 1, 1:, :]
    assert np.array_equal(y[0, 0], want0)
    assert np.array_equal(y[0, 1], want1)


def test_linearity_in_x_and_w():
    x1, w1 = make_inputs(2, 4, 8, 8, 3, 3, 3, seed=5)
    x2, w2 = make_inputs(2, 4, 8, 8, 3, 3, 3, seed=6)
    # use dyadic scalars so that a*x1+b*x2 is exactly representable in fp32 for these draws
    a, b = 0.5, 2.0
    xs = (a * x1.astype(np.float64) + b * x2.astype(np.float64))
    xs32 = xs.astype(np.float32)
    y = conv_ref(xs32, w1, 1, 1)
    want = a * conv_ref(x1, w1, 1, 1) + b * conv_ref(x2, w1, 1, 1)
    # the fp32 cast of xs perturbs it by <= 2^-24 relative; allow for that
    assert np.max(np.abs(y - want)) <= 1e-5 * np.max(np.abs(want))
    ws32 = (a * w1.astype(np.float64) + b * w2.astype(np.float64)).astype(np.float32)
    y2 = conv_ref(x1, ws32, 1, 1)
    want2 = a * conv_ref(x1, w1, 1, 1) + b * conv_ref(x1, w2, 1, 1)
    assert np.max(np.abs(y2 - want2)) <= 1e-5 * np.max(np.abs(want2))


def test_all_ones_counts():
    C = 5
    x = np.ones((1, C, 6, 7), dtype=np.float32)
    w = np.ones((2, C, 3, 3), dtype=np.float32)
    y = conv_ref(x, w, 1, 1)
    assert y[0, 0, 2, 3] == 9 * C and y[0, 1, 0, 3] == 6 * C and y[0, 0, 3, 0] == 6 * C
    for p, q in ((0, 0), (0, 6), (5, 0), (5, 6)):
        assert y[0, 1, p, q] == 4 * C
    assert y.sum() == 2 * C * ((6 * 7) * 9 - 2 * 3 * 7 - 2 * 3 * 6 + 4)


def test_one_by_one_is_a_matrix_product():
    x, w = make_inputs(3, 6, 5, 4, 7, 1, 1, seed=8)
    y = conv_ref(x, w, 1, 0)
    Wm = w.reshape(7, 6).astype(np.float64)
    for n in range(3):
        want = Wm @ x[n].reshape(6, 20).astype(np.float64)
        assert np.allclose(y[n].reshape(7, 20), want, rtol=1e-14, atol=1e-14)


@pytest.mark.parametrize("C,HW,K,R,stride,pad,P", [
    (3, 227, 96, 11, 4, 0, 55), (96, 27, 256, 5, 1, 2, 27), (256, 13, 384, 3, 1, 1, 13), (384, 13, 256, 3, 1, 1, 13)])
def test_table2_output_extents(C, HW, K, R, stride, pad, P):
    # The AlexNet rows of Table 2 (Sec. 7.2) with the floor formula give the familiar 55/27/13/13.
    assert out_extent(HW, HW, R, R, stride, pad) == (P, P)


@pytest.mark.parametrize("N,C,H,W,K,R,S,stride,pad", [
    (2, 3, 35, 35, 4, 11, 11, 4, 0),     # down-scaled AlexNet conv1
    (2, 6, 27, 27, 5, 5, 5, 1, 2),       # conv2
    (2, 8, 13, 13, 6, 3, 3, 1, 1),       # conv3/4
    (1, 4, 10, 12, 3, 3, 3, 2, 1),
    (1, 2, 9, 9, 2, 2, 3, 1, 0),
])
def test_against_torch_cpu_conv2d_fp64(N, C, H, W, K, R, S, stride, pad):
    torch = pytest.importorskip("torch")
    x, w = make_inputs(N, C, H, W, K, R, S, seed=11)
    y = conv_ref(x, w, stride, pad)
    want = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                      stride=stride, padding=pad).numpy()
    assert y.shape == want.shape
    assert np.allclose(y, want, rtol=1e-12, atol=1e-12)


def test_points_agree_with_full_layer():
    x, w = make_inputs(3, 5, 9, 11, 4, 3, 3, seed=12)
    y = conv_ref(x, w, 2, 1)
    N, K, P, Q = y.shape
    idx = sample_output_indices(N, K, P, Q, 64, seed=1)
    pts = conv_ref_points(x, w, idx, 2, 1)
    assert np.array_equal(pts, y[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]])


def test_rejects_bad_arguments():
    x, w = make_inputs(1, 2, 4, 4, 2, 3, 3, seed=1)
    with pytest.raises(ValueError):
        conv_ref(x, w[:, :1], 1, 1)
    with pytest.raises(ValueError):
        conv_ref(x[:, :, :2, :2], w, 1, 0)
