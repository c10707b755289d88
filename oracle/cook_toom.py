"""Exact-rational Winograd / Cook-Toom transform matrices.  TEST INFRASTRUCTURE ONLY.

Follows the Winograd generator of Section 3.3.1 item (3): the interpolation
points are the roots of  x (x-f)(x+f)(x-2f)(x+2f)...  , f = 1/2 by default.
F(n, k) needs alpha - 1 = n + k - 2 finite points and the point at infinity, so
the sequence 0, +f, -f, +2f, -2f, ... is cut after alpha - 1 entries (the
printed last factor, which would give one point too many for even alpha and a
half-integer multiple otherwise, is read this way).

Construction (Toom-Cook polynomial product, transposed into a correlation):
with finite points p_0..p_{alpha-2},
    M(x)   = prod_m (x - p_m)
    M_j(x) = prod_{m != j} (x - p_m)
    N_j    = M_j(p_j)
a polynomial s of degree alpha-1 is recovered from its samples by
    s(x) = s_inf * M(x) + sum_j s(p_j) * M_j(x) / N_j .
Evaluating the two factor polynomials at the points, multiplying samplewise and
interpolating gives a linear convolution; its transpose is the correlation
    y = A^T [ (G g) (.) (B^T d) ],   y_i = sum_j d_{i+j} g_j
with
    A^T[i][j] = p_j^i (j < alpha-1),   A^T[i][alpha-1] = [i == n-1]
    G[j][l]   = p_j^l / N_j,           G[alpha-1][l]   = [l == k-1]
    B^T[j][t] = coeff_t(M_j),          B^T[alpha-1][t] = coeff_t(M)
(the division by N_j may sit in G or in B^T; it is put in G here).

Everything is ``fractions.Fraction``; nothing is rounded.
"""
from __future__ import annotations

from fractions import Fraction
from typing import List, Sequence, Tuple

Matrix = List[List[Fraction]]


def points(alpha: int, f: Fraction = Fraction(1, 2)) -> List[Fraction]:
    """The alpha-1 finite interpolation points 0, +f, -f, +2f, -2f, ..."""
    f = Fraction(f)
    pts = [Fraction(0)]
    m = 1
    while len(pts) < alpha - 1:
        pts.append(m * f)
        if len(pts) < alpha - 1:
            pts.append(-m * f)
        m += 1
    return pts[: alpha - 1]


def _poly_mul_linear(poly: List[Fraction], root: Fraction) -> List[Fraction]:
    """poly(x) * (x - root), coefficients in ascending order."""
    out = [Fraction(0)] * (len(poly) + 1)
    for t, c in enumerate(poly):
        out[t + 1] += c
        out[t] -= root * c
    return out


def _poly_from_roots(roots: Sequence[Fraction]) -> List[Fraction]:
    poly = [Fraction(1)]
    for r in roots:
        poly = _poly_mul_linear(poly, r)
    return poly


def matrices(n: int, k: int, f: Fraction = Fraction(1, 2)) -> Tuple[Matrix, Matrix, Matrix]:
    """Return (A^T  n x alpha,  G  alpha x k,  B^T  alpha x alpha) for F(n, k)."""
    if n < 1 or k < 1:
        raise ValueError("n and k must be positive")
    alpha = n + k - 1
    p = points(alpha, f)
    fin = alpha - 1
    AT = [[Fraction(0)] * alpha for _ in range(n)]
    G = [[Fraction(0)] * k for _ in range(alpha)]
    BT = [[Fraction(0)] * alpha for _ in range(alpha)]
    for j in range(fin):
        others = [p[m] for m in range(fin) if m != j]
        Mj = _poly_from_roots(others)            # degree alpha-2
        Nj = Fraction(1)
        for q in others:
            Nj *= (p[j] - q)
        for i in range(n):
            AT[i][j] = p[j] ** i
        for l in range(k):
            G[j][l] = (p[j] ** l) / Nj
        for t, c in enumerate(Mj):
            BT[j][t] = c
    Mfull = _poly_from_roots(p)                  # degree alpha-1
    AT[n - 1][alpha - 1] = Fraction(1)
    G[alpha - 1][k - 1] = Fraction(1)
    for t, c in enumerate(Mfull):
        BT[alpha - 1][t] = c
    return AT, G, BT


def correlate_via_transforms(AT: Matrix, G: Matrix, BT: Matrix, g: Sequence[Fraction], d: Sequence[Fraction]):
    """A^T [ (G g) (.) (B^T d) ] in exact arithmetic."""
    alpha = len(BT)
    Gg = [sum(G[j][l] * g[l] for l in range(len(g))) for j in range(alpha)]
    Bd = [sum(BT[j][t] * d[t] for t in range(alpha)) for j in range(alpha)]
    had = [Gg[j] * Bd[j] for j in range(alpha)]
    return [sum(AT[i][j] * had[j] for j in range(alpha)) for i in range(len(AT))]


def to_float(M: Matrix):
    import numpy as np
    return np.array([[float(v) for v in row] for row in M], dtype=np.float64)
