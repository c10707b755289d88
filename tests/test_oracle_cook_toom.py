"""Pins for the exact-rational transform generator (oracle/cook_toom.py)."""
from fractions import Fraction as Fr

import os

import numpy as np
import pytest

from oracle import cook_toom

NK = [(n, k) for k in (2, 3, 4, 5, 7) for n in range(1, 9) if n + k - 1 <= 10]


@pytest.mark.parametrize("n,k", NK)
@pytest.mark.parametrize("f", [Fr(1, 2), Fr(1), Fr(3, 7)])
def test_exact_identity_on_all_basis_pairs(n, k, f):
    """A^T[(G e_a) (.) (B^T e_b)]_i == [b == i + a]; bilinearity makes the basis pairs sufficient."""
    AT, G, BT = cook_toom.matrices(n, k, f)
    alpha = n + k - 1
    assert len(AT) == n and len(AT[0]) == alpha
    assert len(G) == alpha and len(G[0]) == k
    assert len(BT) == alpha and len(BT[0]) == alpha
    for a in range(k):
        g = [Fr(int(l == a)) for l in range(k)]
        for bb in range(alpha):
            d = [Fr(int(t == bb)) for t in range(alpha)]
            y = cook_toom.correlate_via_transforms(AT, G, BT, g, d)
            for i in range(n):
                assert y[i] == (1 if bb == i + a else 0), (n, k, a, bb, i)


def test_identity_on_random_rationals_is_correlation_not_convolution():
    n, k = 4, 3
    AT, G, BT = cook_toom.matrices(n, k)
    g = [Fr(3, 5), Fr(-2, 7), Fr(11, 3)]
    d = [Fr(i * i - 3, i + 2) for i in range(n + k - 1)]
    y = cook_toom.correlate_via_transforms(AT, G, BT, g, d)
    assert y == [sum(d[i + j] * g[j] for j in range(k)) for i in range(n)]
    flipped = [sum(d[i + j] * g[k - 1 - j] for j in range(k)) for i in range(n)]
    assert y != flipped


GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_matrices(name):
    """AT, G, BT as lists of rows of Fractions from a tests/golden/*.txt fixture."""
    mats, cur = {}, None
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line in ("AT", "G", "BT"):
            cur = mats.setdefault(line, [])
        else:
            cur.append([Fr(t) for t in line.split()])
    return mats["AT"], mats["G"], mats["BT"]


def test_point_sequence():
    assert cook_toom.points(4) == [0, Fr(1, 2), Fr(-1, 2)]
    assert cook_toom.points(6) == [0, Fr(1, 2), Fr(-1, 2), 1, -1]
    assert cook_toom.points(5) == [0, Fr(1, 2), Fr(-1, 2), 1]            # odd alpha: last point unpaired
    assert cook_toom.points(8) == [0, Fr(1, 2), Fr(-1, 2), 1, -1, Fr(3, 2), Fr(-3, 2)]
    assert cook_toom.points(4, Fr(1)) == [0, 1, -1]
    for a in range(2, 12):
        p = cook_toom.points(a)
        assert len(p) == a - 1 and len(set(p)) == a - 1


def test_f23_worked_values_half_points():
    """F(2,3), points (0, 1/2, -1/2, inf), worked by hand from the interpolation formula:
    M_0 = x^2 - 1/4, N_0 = -1/4; M_1 = x^2 + x/2, N_1 = 1/2; M_2 = x^2 - x/2, N_2 = 1/2; M = x^3 - x/4."""
    AT, G, BT = cook_toom.matrices(2, 3, Fr(1, 2))
    AT_w, G_w, BT_w = read_matrices("winograd_F23_half_points.txt")
    assert AT == AT_w and G == G_w and BT == BT_w
    h, q = Fr(1, 2), Fr(1, 4)
    assert AT == [[1, 1, 1, 0], [0, h, -h, 1]] and BT[0] == [-q, 0, 1, 0]      # the fixture is what the docstring says


def _rank_one_terms(AT, G, BT):
    """The decomposition's rank-one terms a_j (x) g_j (x) b_j: what is unique under row/column rescaling."""
    AT, G, BT = (np.array([[float(v) for v in r] for r in m]) for m in (AT, G, BT))
    return np.einsum("ij,jl,jt->jilt", AT, G, BT)


def test_f23_unit_points_equal_the_classic_matrices_up_to_scaling():
    # The widely published F(2,3) matrices for points (0, 1, -1, inf) (Lavin & Gray, "Fast algorithms
    # for convolutional neural networks", the work the paper cites for Winograd convolution).
    AT_c, G_c, BT_c = read_matrices("winograd_F23_unit_points.txt")
    AT, G, BT = cook_toom.matrices(2, 3, Fr(1))
    np.testing.assert_allclose(_rank_one_terms(AT, G, BT), _rank_one_terms(AT_c, G_c, BT_c), atol=0)


def test_f43_unit_points_equal_the_classic_matrices_up_to_scaling():
    # F(4,3) for points (0, 1, -1, 2, -2, inf) from the same publication.
    AT_c, G_c, BT_c = read_matrices("winograd_F43_unit_points.txt")
    AT, G, BT = cook_toom.matrices(4, 3, Fr(1))
    np.testing.assert_allclose(_rank_one_terms(AT, G, BT), _rank_one_terms(AT_c, G_c, BT_c), atol=1e-15)


def test_half_points_are_more_accurate_in_float32_than_unit_points():
    """The stated purpose of f: F(6,3) evaluated in float32 loses far less with f = 1/2 than with f = 1."""
    rng = np.random.default_rng(0)
    n, k = 6, 3
    g = rng.normal(0, 1, (2000, k))
    d = rng.uniform(-1, 1, (2000, n + k - 1))
    ref = np.stack([sum(d[:, i + j] * g[:, j] for j in range(k)) for i in range(n)], axis=1)

    def err(f):
        AT, G, BT = (cook_toom.to_float(m).astype(np.float32) for m in cook_toom.matrices(n, k, f))
        y = ((g.astype(np.float32) @ G.T) * (d.astype(np.float32) @ BT.T)) @ AT.T
        return np.max(np.abs(y - ref)) / np.max(np.abs(ref))

    assert err(Fr(1, 2)) < 0.2 * err(Fr(1))


def _float32_winograd_error(n, k, f, C=64, T=48, seed=7):
    """max|err| / max|ref| of one Winograd tile computation carried out in float32 with the exact matrices rounded once,
    against the float64 correlation of the same float32 data: what any float32 implementation of F(n, k) is up against."""
    AT, G, BT = cook_toom.matrices(n, k, Fr(f).limit_denominator(1000))
    a = n + k - 1
    AT32, G32, BT32 = (np.array([[float(v) for v in row] for row in m], np.float32) for m in (AT, G, BT))
    rng = np.random.default_rng(seed)
    d = rng.uniform(-1, 1, (T, C, a, a)).astype(np.float32)
    g = rng.normal(0, np.sqrt(2.0 / (k * k * C)), (C, k, k)).astype(np.float32)
    U = np.einsum("ik,ckl,jl->cij", G32, g, G32).astype(np.float32)
    V = np.einsum("ik,tckl,jl->tcij", BT32, d, BT32).astype(np.float32)
    M = np.einsum("cij,tcij->tij", U, V).astype(np.float32)
    Y = np.einsum("ik,tkl,jl->tij", AT32, M, AT32).astype(np.float32)
    ref = np.zeros((T, n, n))
    for i in range(n):
        for j in range(n):
            ref[:, i, j] = np.einsum("tckl,ckl->t", d[:, :, i:i + k, j:j + k].astype(np.float64), g.astype(np.float64))
    return float(np.abs(Y - ref).max() / np.abs(ref).max())


def test_float32_error_bounds_the_usable_tile_sizes():
    """Why the library stops at alpha = n + k - 1 = 10: in float32 the generated transforms keep the 1e-3 bound up to
    alpha = 10 and lose it at alpha = 11, for the paper's f = 0.5 and for closer points alike; and why it spaces the
    points 0.425 apart for alpha = 9, 10 when asked to choose (several times less error than 0.5, the reverse at 8)."""
    for n, k in ((6, 3), (4, 5), (2, 7)):
        assert _float32_winograd_error(n, k, 0.5) < 1e-4                      # alpha = 8
    for n, k in ((7, 3), (8, 3), (6, 5), (4, 7)):                               # alpha = 9, 10
        e5, e4 = _float32_winograd_error(n, k, 0.5), _float32_winograd_error(n, k, 0.425)
        assert e5 < 1e-3 and e4 < 3e-4 and e4 < 0.7 * e5
    for n, k in ((9, 3), (5, 7), (10, 3)):                                     # alpha = 11, 12
        assert _float32_winograd_error(n, k, 0.5) > 5e-3
        assert _float32_winograd_error(n, k, 0.425) > 1e-3
    assert _float32_winograd_error(6, 3, 0.5) < _float32_winograd_error(6, 3, 0.425)
