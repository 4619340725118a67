"""TEST INFRASTRUCTURE ONLY: CPU oracle for the Winograd convolution F(e x e, r x r).

Follows the paper's four steps (Sec. 2.3 "Winograd Algorithm" and the four-step DAG of
Sec. 4.3) in the paper's notation:

  step 1  P_i = B I_i B^T   (input tile transform)      J_k = L K_k L^T   (kernel transform)
  step 2  Lambda_{i,k} = P_i (.) J_k                     (element-wise product, per channel)
  step 3  Pi_{i,k} = sum over channels of Lambda_{i,k}   (channel summation)
  step 4  e x e outputs = A Pi_{i,k} A^T                 (output transform)

The paper never prints the entries of A, B and L.  They are derived here in exact rational
arithmetic from the defining property of a minimal 1-D filtering algorithm,

    y_i = sum_k d_{i+k} g_k  ==  sum_j A[i][j] * (L g)_j * (B d)_j      for all d, g,

with A and L fixed by a choice of interpolation points (Toom-Cook construction) and B obtained
by solving that identity as a linear system.  Everything after the matrices is fp64 numpy.

Shapes: A is e x n, B is n x n, L is n x r, with n = e + r - 1.
No code is shared with the GPU library.
"""
from fractions import Fraction

import numpy as np

INF = "inf"

# Interpolation points.  Any distinct set works in exact arithmetic; small magnitudes keep
# the fp32 error of the e = 4 variant low.
DEFAULT_POINTS = {
    2: [0, 1, -1, INF],
    3: [0, 1, -1, 2, INF],
    4: [0, 1, -1, 2, -2, INF],
    6: [0, 1, -1, 2, -2, Fraction(1, 2), Fraction(-1, 2), INF],
}


def _solve_exact(rows, rhs):
    """Solve a consistent, possibly over-determined linear system over the rationals."""
    m = [list(r) + [b] for r, b in zip(rows, rhs)]
    ncol = len(rows[0])
    piv_rows = []
    rank = 0
    for col in range(ncol):
        sel = None
        for i in range(rank, len(m)):
            if m[i][col] != 0:
                sel = i
                break
        if sel is None:
            raise ValueError("system is rank deficient: interpolation points not distinct?")
        m[rank], m[sel] = m[sel], m[rank]
        pv = m[rank][col]
        m[rank] = [v / pv for v in m[rank]]
        for i in range(len(m)):
            if i != rank and m[i][col] != 0:
                f = m[i][col]
                m[i] = [a - f * b for a, b in zip(m[i], m[rank])]
        piv_rows.append(rank)
        rank += 1
    for i in range(rank, len(m)):
        if m[i][ncol] != 0:
            raise ValueError("system is inconsistent")
    return [m[i][ncol] for i in range(ncol)]


def winograd_matrices(e, r=3, points=None):
    """Exact (A, B, L) for F(e, r) as nested lists of Fraction."""
    n = e + r - 1
    pts = list(DEFAULT_POINTS[e] if points is None else points)
    if len(pts) != n or pts.count(INF) != 1 or pts[-1] != INF:
        raise ValueError("need n-1 finite points followed by INF")
    fin = [Fraction(p) for p in pts[:-1]]
    if len(set(fin)) != len(fin):
        raise ValueError("points must be distinct")
    # A: evaluation of a degree-(e-1) polynomial at the points, transposed.
    A = [[fin[j] ** i for j in range(n - 1)] + [Fraction(int(i == e - 1))] for i in range(e)]
    # L: evaluation of the degree-(r-1) kernel polynomial, each row divided by the product
    # of point differences (the Lagrange denominator); the point at infinity takes the
    # leading coefficient.
    L = []
    for j in range(n - 1):
        den = Fraction(1)
        for l in range(n - 1):
            if l != j:
                den *= fin[j] - fin[l]
        L.append([fin[j] ** k / den for k in range(r)])
    L.append([Fraction(int(k == r - 1)) for k in range(r)])
    # B: solve  sum_j A[i][j] L[j][k] B[j][l] = [l == i + k]  column by column.
    rows = [[A[i][j] * L[j][k] for j in range(n)] for i in range(e) for k in range(r)]
    B = [[None] * n for _ in range(n)]
    for l in range(n):
        rhs = [Fraction(int(l == i + k)) for i in range(e) for k in range(r)]
        col = _solve_exact(rows, rhs)
        for j in range(n):
            B[j][l] = col[j]
    return A, B, L


def _to_f64(M):
    return np.array([[float(v) for v in row] for row in M], dtype=np.float64)


def winograd_conv(x, w, e, pad=1, points=None):
    """Winograd F(e x e, r x r) convolution of a batch, stride 1, zero padding `pad`; fp64 result.

    x: [N][C][H][W], w: [K][C][r][r]; returns y: [N][K][Ho][Wo] with Ho = H + 2 pad - r + 1.
    The output plane is cut into ceil(Ho/e) x ceil(Wo/e) sub-domains of e x e outputs; tiles
    hanging over the edge read zeros and only their valid outputs are kept.
    """
    x = np.asarray(x, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    N, C, H, W = x.shape
    K, C2, r, r2 = w.shape
    if C2 != C or r != r2:
        raise ValueError("shape mismatch")
    n = e + r - 1
    A, B, L = (_to_f64(M) for M in winograd_matrices(e, r, points))
    Ho, Wo = H + 2 * pad - r + 1, W + 2 * pad - r + 1
    th, tw = -(-Ho // e), -(-Wo // e)
    # zero-extended input: `pad` on the top/left, enough on the bottom/right for the last tile
    xe = np.zeros((N, C, th * e + r - 1, tw * e + r - 1), dtype=np.float64)
    xe[:, :, pad:pad + H, pad:pad + W] = x
    # step 1b: J_k = L K_k L^T for every kernel and channel
    J = np.einsum("ar,kcrs,bs->kcab", L, w, L)
    y = np.zeros((N, K, th * e, tw * e), dtype=np.float64)
    for ti in range(th):
        for tj in range(tw):
            I = xe[:, :, ti * e:ti * e + n, tj * e:tj * e + n]          # sliding input tensor
            P = np.einsum("ai,ncij,bj->ncab", B, I, B)                   # step 1a
            Lam = P[:, None, :, :, :] * J[None, :, :, :, :]              # step 2  [N][K][C][n][n]
            Pi = Lam.sum(axis=2)                                         # step 3
            y[:, :, ti * e:(ti + 1) * e, tj * e:(tj + 1) * e] = \
                np.einsum("ia,nkab,jb->nkij", A, Pi, A)                  # step 4
    return y[:, :, :Ho, :Wo]
