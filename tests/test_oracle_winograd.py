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
