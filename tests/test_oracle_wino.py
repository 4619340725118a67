"""Pins for the Winograd oracle (oracle/wino_oracle.py): the transform matrices are checked in
exact rational arithmetic against the definition of correlation, and the fp64 Winograd layer is
checked against the direct-convolution oracle.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from oracle.conv_oracle import conv_ref
from oracle.wino_oracle import INF, winograd_conv, winograd_matrices
from paper_2012_15667_amd.inputs import make_inputs


def _mat_vec(M, v):
    return [sum(a * b for a, b in zip(row, v)) for row in M]


@pytest.mark.parametrize("e", [2, 3, 4, 6])
def test_1d_identity_on_basis_vectors_exact(e):
    r = 3
    n = e + r - 1
    A, B, L = winograd_matrices(e, r)
    assert (len(A), len(A[0])) == (e, n) and (len(B), len(B[0])) == (n, n) and (len(L), len(L[0])) == (n, r)
    for di in range(n):
        d = [Fraction(int(i == di)) for i in range(n)]
        Bd = _mat_vec(B, d)
        for gi in range(r):
            g = [Fraction(int(i == gi)) for i in range(r)]
            Lg = _mat_vec(L, g)
            y = _mat_vec(A, [a * b for a, b in zip(Lg, Bd)])
            want = [sum(d[i + k] * g[k] for k in range(r)) for i in range(e)]    # y_i = sum_k d_{i+k} g_k
            assert y == want


@pytest.mark.parametrize("e", [2, 3, 4, 6])
def test_2d_tile_exact_small_integers(e):
    """A (L g L^T (.) B d B^T) A^T equals the e x e correlation outputs of one tile, exactly."""
    r, n = 3, e + 2
    A, B, L = winograd_matrices(e, r)
    rng = np.random.default_rng(5)
    d = [[Fraction(int(v)) for v in row] for row in rng.integers(-5, 6, size=(n, n))]
    g = [[Fraction(int(v)) for v in row] for row in rng.integers(-5, 6, size=(r, r))]

    def mm(X, Y):
        return [[sum(X[i][k] * Y[k][j] for k in range(len(Y))) for j in range(len(Y[0]))] for i in range(len(X))]

    def tr(X):
        return [list(c) for c in zip(*X)]

    P = mm(mm(B, d), tr(B))
    J = mm(mm(L, g), tr(L))
    Lam = [[P[i][j] * J[i][j] for j in range(n)] for i in range(n)]
    Y = mm(mm(A, Lam), tr(A))
    for i in range(e):
        for j in range(e):
            assert Y[i][j] == sum(d[i + a][j + b] * g[a][b] for a in range(r) for b in range(r))


def test_multiplication_counts():
    # F(e x e, 3 x 3) spends (e+2)^2 multiplications per tile where the definition spends 9 e^2
    for e, want in ((2, 16), (3, 25), (4, 36), (6, 64)):
        A, B, L = winograd_matrices(e)
        assert len(B) ** 2 == want < 9 * e * e


def test_input_transform_is_integer_valued_for_integer_points():
    for e in (2, 3, 4):        # e = 6 uses the points +-1/2
        _, B, _ = winograd_matrices(e)
        assert all(v.denominator == 1 for row in B for v in row)


def test_other_points_give_the_same_layer():
    x, w = make_inputs(1, 3, 8, 8, 2, 3, 3, seed=21)
    y1 = winograd_conv(x, w, 2)
    y2 = winograd_conv(x, w, 2, points=[0, 2, Fraction(-1, 2), INF])
    assert np.allclose(y1, y2, rtol=1e-12, atol=1e-12)


def test_rejects_repeated_points():
    with pytest.raises(ValueError):
        winograd_matrices(2, 3, points=[0, 1, 1, INF])


@pytest.mark.parametrize("e,N,C,H,W,K", [
    (2, 2, 5, 8, 8, 4),
    (2, 1, 3, 7, 9, 2),        # ragged: odd extents
    (4, 2, 6, 14, 14, 5),      # ragged: 14 = 3.5 tiles of 4
    (4, 1, 4, 13, 13, 3),      # AlexNet conv3/4 extent
    (4, 1, 2, 16, 12, 2),
    (4, 1, 3, 3, 5, 2),        # smaller than one tile
    (3, 2, 4, 9, 12, 3),
    (3, 1, 3, 14, 13, 2),      # ragged: neither extent a multiple of 3
    (6, 1, 3, 12, 18, 2),
    (6, 2, 2, 14, 13, 3),      # ragged: 14 = 2.33 tiles of 6
    (6, 1, 2, 4, 5, 2),        # smaller than one tile
])
def test_winograd_layer_matches_direct_oracle_fp64(e, N, C, H, W, K):
    x, w = make_inputs(N, C, H, W, K, 3, 3, seed=31 + e)
    y = winograd_conv(x, w, e, pad=1)
    ref = conv_ref(x, w, 1, 1)
    assert y.shape == ref.shape
    assert np.max(np.abs(y - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_winograd_pad0():
    x, w = make_inputs(1, 2, 10, 10, 2, 3, 3, seed=40)
    assert np.allclose(winograd_conv(x, w, 4, pad=0), conv_ref(x, w, 1, 0), rtol=1e-12, atol=1e-12)
