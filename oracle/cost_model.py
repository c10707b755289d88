"""Analytic scheme-selection cost.  TEST INFRASTRUCTURE ONLY.

Section 3.2, "Computation scheme selection":
  * k = 1                       -> matrix multiplication
  * k > 1: per-block arithmetic cost of Winograd with output tile n
        C(n) = 2 i_c (n+k-1)^3 + i_c o_c (n+k-1)^2 + n (n+k-1)(2n+k-1)
    n_hat = argmin_n C(n);  n_hat = 1 -> sliding window, else F(n_hat x n_hat, k x k).

Reading used here (the printed C(n) is the cost of ONE block and grows with n,
so minimising it as printed always returns 1): the quantity minimised is the
cost of the whole output plane, ceil(o_h/n) * ceil(o_w/n) * C(n), over
1 <= n with n + k - 1 <= alpha_max (the paper gives no upper bound for n; 8 is
this build's default).  Ties go to the smaller n.

Section 3.3.2: Strassen recursion on [n,k] x [k,m] continues only while
    m n k - 7 (m/2)(n/2)(k/2)  >  4 (m/2)(k/2) + 4 (n/2)(k/2) + 7 (m/2)(n/2).
"""
from __future__ import annotations

from fractions import Fraction


def block_cost(n: int, k: int, i_c: int, o_c: int) -> int:
    a = n + k - 1
    return 2 * i_c * a ** 3 + i_c * o_c * a ** 2 + n * a * (2 * n + k - 1)


def plane_cost(n: int, k: int, i_c: int, o_c: int, o_h: int, o_w: int) -> int:
    blocks = -(-o_h // n) * -(-o_w // n)
    return blocks * block_cost(n, k, i_c, o_c)


def best_tile(k: int, i_c: int, o_c: int, o_h: int, o_w: int, alpha_max: int = 8) -> int:
    best_n, best_c = 1, plane_cost(1, k, i_c, o_c, o_h, o_w)
    n = 2
    while n + k - 1 <= alpha_max:
        c = plane_cost(n, k, i_c, o_c, o_h, o_w)
        if c < best_c:
            best_n, best_c = n, c
        n += 1
    return best_n


def scheme(k: int, i_c: int, o_c: int, o_h: int, o_w: int, alpha_max: int = 8) -> str:
    if k == 1:
        return "gemm"
    n_hat = best_tile(k, i_c, o_c, o_h, o_w, alpha_max)
    return "sliding" if n_hat == 1 else f"F({n_hat},{k})"


def strassen_should_recurse(n: int, k: int, m: int) -> bool:
    h = Fraction(1, 2)
    saved = m * n * k - 7 * (m * h) * (n * h) * (k * h)
    extra = 4 * (m * h) * (k * h) + 4 * (n * h) * (k * h) + 7 * (m * h) * (n * h)
    return saved > extra
