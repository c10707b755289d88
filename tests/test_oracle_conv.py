"""Pins for the float64 direct-convolution oracle (oracle/conv_direct.c).

None of these re-types the oracle's own loop nest as the expected value in a way
that could share its mistakes: they are (i) an independently indexed brute-force
in pure Python over an explicitly padded array, (ii) closed forms, (iii) the
k = 1 special case against a library matrix product, (iv) PyTorch's float64 CPU
convolution (a library routine for the same definition), (v) linearity and
shift properties.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
from conv_workloads import small_parity_layers, draw


def brute_force(x, w, b, stride, pad, dil):
    """Seven nested Python loops over an explicitly zero-padded copy of x."""
    N, C, H, W = x.shape
    K, _, kh, kw = w.shape
    xp = np.zeros((N, C, H + 2 * pad, W + 2 * pad), dtype=np.float64)
    xp[:, :, pad:pad + H, pad:pad + W] = x
    Ho = (H + 2 * pad - dil * (kh - 1) - 1) // stride + 1
    Wo = (W + 2 * pad - dil * (kw - 1) - 1) // stride + 1
    y = np.zeros((N, K, Ho, Wo), dtype=np.float64)
    for n in range(N):
        for k in range(K):
            for oy in range(Ho):
                for ox in range(Wo):
                    s = float(b[k]) if b is not None else 0.0
                    for c in range(C):
                        for r in range(kh):
                            for q in range(kw):
                                s += xp[n, c, oy * stride + r * dil, ox * stride + q * dil] * float(w[k, c, r, q])
                    y[n, k, oy, ox] = s
    return y


TINY = [
    # N, C, H, W, K, k, stride, pad, dil
    (1, 1, 4, 4, 1, 1, 1, 0, 1),
    (2, 3, 6, 5, 2, 3, 1, 1, 1),
    (1, 2, 6, 6, 3, 2, 1, 0, 1),
    (2, 2, 6, 6, 2, 5, 1, 2, 1),
    (1, 3, 6, 6, 2, 3, 2, 1, 1),
    (1, 2, 6, 6, 2, 3, 1, 2, 2),
    (2, 3, 5, 6, 3, 3, 2, 0, 1),
    (1, 2, 6, 6, 2, 2, 2, 1, 2),
]


@pytest.mark.parametrize("shape", TINY)
def test_oracle_matches_brute_force(shape):
    N, C, H, W, K, k, s, p, d = shape
    rng = np.random.default_rng(1234 + sum(shape))
    x = rng.uniform(-1, 1, (N, C, H, W)).astype(np.float32)
    w = rng.normal(0, 1, (K, C, k, k)).astype(np.float32)
    b = rng.uniform(-1, 1, (K,)).astype(np.float32)
    y = oracle.conv2d(x, w, b, stride=s, pad=p, dil=d)
    ref = brute_force(x, w, b, s, p, d)
    assert y.shape == ref.shape
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)


def test_all_ones_counts_in_bounds_taps():
    # x = 1, w = 1, b = 0  =>  y = C * (number of kernel taps that fall inside the image)
    N, C, H, W, K, k, pad = 1, 3, 7, 6, 2, 3, 1
    x = np.ones((N, C, H, W), np.float32)
    w = np.ones((K, C, k, k), np.float32)
    y = oracle.conv2d(x, w, None, stride=1, pad=pad)
    assert y.shape == (N, K, H, W)
    for oy, ox in itertools.product(range(H), range(W)):
        rows = sum(1 for r in range(k) if 0 <= oy - pad + r < H)
        cols = sum(1 for s in range(k) if 0 <= ox - pad + s < W)
        assert y[0, 0, oy, ox] == C * rows * cols
        assert y[0, 1, oy, ox] == C * rows * cols
    assert y[0, 0, 3, 3] == C * k * k          # interior
    assert y[0, 0, 0, 0] == C * 4              # corner sees a 2x2 patch


def test_unit_impulse_reproduces_unflipped_kernel():
    # x = delta at (cy, cx) in channel c0  =>  y[k, oy, ox] = w[k, c0, cy - oy + pad, cx - ox + pad]
    C, K, k, pad, H, W = 2, 3, 3, 1, 7, 7
    rng = np.random.default_rng(7)
    w = rng.normal(0, 1, (K, C, k, k)).astype(np.float32)
    x = np.zeros((1, C, H, W), np.float32)
    c0, cy, cx = 1, 3, 4
    x[0, c0, cy, cx] = 1.0
    y = oracle.conv2d(x, w, None, stride=1, pad=pad)
    for kk in range(K):
        for oy in range(H):
            for ox in range(W):
                r, s = cy - oy + pad, cx - ox + pad
                expect = float(w[kk, c0, r, s]) if (0 <= r < k and 0 <= s < k) else 0.0
                assert y[0, kk, oy, ox] == expect
    # cross-correlation, not convolution: the tap that meets the impulse at output (cy-1, cx-1)
    # is w[.., 2, 2], the bottom-right one.
    assert y[0, 0, cy - 1, cx - 1] == float(w[0, c0, 2, 2])


def test_pointwise_equals_matrix_product():
    rng = np.random.default_rng(11)
    N, C, H, W, K = 3, 19, 5, 7, 23
    x = rng.uniform(0, 1, (N, C, H, W)).astype(np.float32)
    w = rng.normal(0, 1, (K, C, 1, 1)).astype(np.float32)
    b = rng.uniform(-0.1, 0.1, (K,)).astype(np.float32)
    y = oracle.conv2d(x, w, b)
    W2 = w.reshape(K, C).astype(np.float64)
    for n in range(N):
        ref = W2 @ x[n].reshape(C, H * W).astype(np.float64) + b.astype(np.float64)[:, None]
        np.testing.assert_allclose(y[n].reshape(K, H * W), ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("layer", small_parity_layers(), ids=lambda l: l.name)
def test_against_torch_float64_conv(layer):
    x, w, b = draw(layer)
    y = oracle.conv2d(x, w, b, stride=layer.stride, pad=layer.pad, dil=layer.dil)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     torch.from_numpy(b).double(), stride=layer.stride,
                                     padding=layer.pad, dilation=layer.dil).numpy()
    assert y.shape == ref.shape == (layer.n, layer.c_out, layer.h_out, layer.w_out)
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-11)


def test_linearity_and_shift():
    rng = np.random.default_rng(5)
    x1 = rng.uniform(-1, 1, (1, 3, 9, 9)).astype(np.float32)
    x2 = rng.uniform(-1, 1, (1, 3, 9, 9)).astype(np.float32)
    w = rng.normal(0, 1, (4, 3, 3, 3)).astype(np.float32)
    # exact float32 sums so that widening commutes with the addition
    x1 = np.round(x1 * 256) / 256
    x2 = np.round(x2 * 256) / 256
    y1 = oracle.conv2d(x1, w, None, pad=0)
    y2 = oracle.conv2d(x2, w, None, pad=0)
    y12 = oracle.conv2d((x1 + x2).astype(np.float32), w, None, pad=0)
    np.testing.assert_allclose(y12, y1 + y2, rtol=0, atol=1e-12)
    # shifting the input by one pixel shifts the valid output by one pixel
    xs = np.zeros_like(x1)
    xs[:, :, 1:, 1:] = x1[:, :, :-1, :-1]
    ys = oracle.conv2d(xs, w, None, pad=0)
    np.testing.assert_allclose(ys[:, :, 1:, 1:], y1[:, :, :-1, :-1], rtol=0, atol=1e-12)


def test_points_variant_agrees_with_full():
    layer = small_parity_layers()[2]
    x, w, b = draw(layer)
    y = oracle.conv2d(x, w, b, stride=layer.stride, pad=layer.pad, dil=layer.dil)
    rng = np.random.default_rng(3)
    coords = np.stack([rng.integers(0, s, 50) for s in y.shape], axis=1)
    got = oracle.conv2d_points(x, w, b, coords, stride=layer.stride, pad=layer.pad, dil=layer.dil)
    np.testing.assert_array_equal(got, y[coords[:, 0], coords[:, 1], coords[:, 2], coords[:, 3]])


def test_rejects_bad_shapes():
    x = np.zeros((1, 1, 2, 2), np.float32)
    w = np.zeros((1, 1, 3, 3), np.float32)
    with pytest.raises(ValueError):
        oracle.conv2d(x, w, None, pad=0)       # kernel larger than the image


def test_error_ratio_metric():
    ref = np.array([1.0, -4.0, 2.0])
    assert oracle.error_ratio(ref, ref) == 0.0
    assert oracle.error_ratio(ref + np.array([0.0, 0.0, 0.4]), ref) == pytest.approx(0.1)
