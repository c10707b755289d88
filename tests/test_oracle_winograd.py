"""The step-by-step float64 Winograd (oracle/winograd.py) must equal the definition (oracle.conv2d)."""
import numpy as np
import pytest

import oracle
from oracle import winograd
from conv_workloads import ConvLayer, draw, BASE_SEED

CASES = [
    # n, k, N, C, H, W, K, pad
    (2, 3, 1, 3, 6, 6, 2, 1),
    (4, 3, 2, 5, 7, 7, 6, 1),      # ragged: 7 = 4 + 3
    (6, 3, 1, 4, 14, 9, 3, 1),     # ragged both ways
    (4, 3, 2, 3, 13, 13, 2, 0),    # no padding
    (2, 5, 1, 3, 11, 15, 4, 2),
    (4, 5, 1, 2, 12, 12, 3, 2),
    (2, 7, 1, 2, 16, 16, 2, 3),
    (3, 2, 2, 3, 9, 9, 2, 0),      # even kernel, odd alpha... F(3,2): alpha = 4
    (5, 3, 1, 2, 10, 10, 2, 1),    # odd alpha = 7: unpaired last point
    (2, 3, 1, 2, 8, 8, 2, 2),      # pad larger than (k-1)/2
]


@pytest.mark.parametrize("case", CASES)
def test_winograd_float64_equals_definition(case):
    n, k, N, C, H, W, K, pad = case
    layer = ConvLayer("t", N, C, H, W, K, k, k, 1, pad, 1, (-1.0, 1.0), BASE_SEED + 77 + sum(case))
    x, w, b = draw(layer)
    ref = oracle.conv2d(x, w, b, stride=1, pad=pad)
    y, st = winograd.winograd_conv2d(x, w, b, n, pad=pad, return_stages=True)
    assert y.shape == ref.shape
    assert oracle.error_ratio(y, ref) < 1e-11
    alpha = n + k - 1
    P = N * -(-layer.h_out // n) * -(-layer.w_out // n)
    assert st["U"].shape == (alpha, alpha, K, C)
    assert st["V"].shape == (alpha, alpha, C, P)
    assert st["M"].shape == (alpha, alpha, K, P)


def test_no_bias():
    layer = ConvLayer("t", 1, 3, 8, 8, 2, 3, 3, 1, 1, 1, (-1.0, 1.0), BASE_SEED + 5)
    x, w, _ = draw(layer)
    ref = oracle.conv2d(x, w, None, pad=1)
    assert oracle.error_ratio(winograd.winograd_conv2d(x, w, None, 4, pad=1), ref) < 1e-12


RECT_CASES = [
    # n, kh, kw, N, C, H, W, K, pad
    (2, 1, 7, 1, 3, 9, 20, 2, (0, 3)),
    (2, 7, 1, 2, 2, 17, 13, 3, (3, 0)),
    (4, 1, 3, 2, 4, 9, 22, 3, (0, 1)),     # ragged along W: 22 = 5*4 + 2
    (6, 3, 1, 1, 2, 20, 5, 2, (1, 0)),     # ragged along H
    (4, 5, 1, 1, 3, 23, 6, 4, (0, 0)),     # no padding
    (3, 1, 2, 1, 2, 6, 11, 2, (0, 0)),     # even kernel
]


@pytest.mark.parametrize("case", RECT_CASES)
def test_single_row_or_column_kernels_equal_definition(case):
    """One-dimensional F(n, k) along the long side, identity along the other: still the plain convolution."""
    n, kh, kw, N, C, H, W, K, pad = case
    layer = ConvLayer("t", N, C, H, W, K, kh, kw, 1, pad, 1, (-1.0, 1.0), BASE_SEED + 177 + n + kh * 7 + kw)
    x, w, b = draw(layer)
    ref = oracle.conv2d(x, w, b, stride=1, pad=pad)
    y, st = winograd.winograd_conv2d(x, w, b, n, pad=pad, return_stages=True)
    assert y.shape == ref.shape
    assert oracle.error_ratio(y, ref) < 1e-11
    ah, aw = (1, n + kw - 1) if kh == 1 else (n + kh - 1, 1)
    th, tw = (layer.h_out, -(-layer.w_out // n)) if kh == 1 else (-(-layer.h_out // n), layer.w_out)
    assert st["U"].shape == (ah, aw, K, C)
    assert st["V"].shape == (ah, aw, C, N * th * tw)
    # along the untransformed side the transforms are the identity: U is G applied to the kernel's one line
    line = w[:, :, 0, :] if kh == 1 else w[:, :, :, 0]
    g = st["G_w"] if kh == 1 else st["G"]
    assert np.allclose(st["U"].reshape(max(ah, aw), K, C), np.einsum("ir,kcr->ikc", g, line), rtol=0, atol=1e-14)


MIXED_CASES = [
    # n, kh, kw, N, C, H, W, K, pad: several taps on both axes, kh != kw
    (2, 3, 5, 1, 3, 10, 12, 2, (1, 2)),
    (4, 5, 2, 2, 2, 14, 9, 3, (0, 0)),      # even taps along W, ragged tiles both ways
    (2, 2, 7, 1, 2, 11, 19, 2, (1, 2)),
    (5, 4, 3, 1, 3, 13, 15, 2, (2, 1)),     # n = 5: alpha 8 x 7
    (3, 7, 4, 1, 2, 16, 9, 2, (3, 0)),      # alpha 9 x 6
]


@pytest.mark.parametrize("case", MIXED_CASES)
def test_kernels_with_different_tap_counts_per_axis_equal_definition(case):
    """k_h x k_w kernels: F(n, k_h) down the columns and F(n, k_w) along the rows is still the plain convolution, and
    U is the two-sided transform of the kernel with the two different G matrices."""
    n, kh, kw, N, C, H, W, K, pad = case
    layer = ConvLayer("t", N, C, H, W, K, kh, kw, 1, pad, 1, (-1.0, 1.0), BASE_SEED + 277 + n + kh * 7 + kw)
    x, w, b = draw(layer)
    ref = oracle.conv2d(x, w, b, stride=1, pad=pad)
    y, st = winograd.winograd_conv2d(x, w, b, n, pad=pad, return_stages=True)
    assert y.shape == ref.shape
    assert oracle.error_ratio(y, ref) < 1e-10
    ah, aw = n + kh - 1, n + kw - 1
    assert st["U"].shape == (ah, aw, K, C) and st["G"].shape == (ah, kh) and st["G_w"].shape == (aw, kw)
    assert st["V"].shape == (ah, aw, C, N * (-(-layer.h_out // n)) * (-(-layer.w_out // n)))
    # a kernel that is an outer product a (x) b transforms into the outer product (G_h a) (x) (G_w b)
    a_vec, b_vec = np.arange(1.0, kh + 1), np.arange(1.0, kw + 1)[::-1]
    w1 = np.broadcast_to(np.outer(a_vec, b_vec), (1, 1, kh, kw)).astype(np.float64)
    _, st1 = winograd.winograd_conv2d(np.zeros((1, 1, H, W)), w1, None, n, pad=pad, return_stages=True)
    assert np.allclose(st1["U"][:, :, 0, 0], np.outer(st["G"] @ a_vec, st["G_w"] @ b_vec), rtol=1e-13, atol=1e-13)
