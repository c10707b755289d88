"""Strassen's algorithm for the large matrix multiplication (Section 3.3.2) on the device.

It reaches the plain product exactly up to rounding order, so the oracle is the definition: a float64 matrix
product (numpy) of the float32 operands.  Tolerance: the 1e-4 of max|D| that the plain fp32 GEMM is held to,
whatever the number of levels (every level adds a few fp32 roundings per element; measured errors are about 1e-6).
"""
import numpy as np
import pytest
import torch

import oracle
from conv_workloads import BASE_SEED, ConvLayer, draw

pytestmark = pytest.mark.gpu


def mnn():
    import paper_2002_12418_amd as m
    return m


@pytest.mark.parametrize("M,R,N,levels", [(64, 32, 96, 1), (256, 256, 256, 1), (256, 256, 256, 2), (512, 384, 640, 2),
                                          (128, 8, 1024, 3), (1024, 1024, 784, 0)])
def test_strassen_against_float64_product(M, R, N, levels):
    m = mnn()
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 31 * M + 7 * R + N + levels))
    At = rng.normal(0, 1, (R, M)).astype(np.float32)          # A stored transposed
    B = rng.uniform(-1, 1, (R, N)).astype(np.float32)
    bias = rng.uniform(-0.1, 0.1, M).astype(np.float32)
    ref = At.astype(np.float64).T @ B.astype(np.float64) + bias.astype(np.float64)[:, None]
    Atd, Bd, bd = (torch.from_numpy(a).cuda() for a in (At, B, bias))
    D = torch.full((M, N), float("nan"), device="cuda")
    with m.StrassenGemm(M, N, R, levels) as sg:
        info = sg.info
        assert info["levels"] == levels and info["launches"] >= 2 * levels + 1
        sg.set_left(Atd)
        sg.run(Bd, D, bd)
        torch.cuda.synchronize()
        got = D.cpu().numpy()
        # a second right operand against the same expanded left one, no bias
        B2 = rng.uniform(-1, 1, (R, N)).astype(np.float32)
        D2 = sg.run(torch.from_numpy(B2).cuda(), torch.empty_like(D))
        torch.cuda.synchronize()
    assert np.isfinite(got).all()
    err = oracle.error_ratio(got, ref)
    print(f"[strassen] {M}x{R}x{N} levels={levels} err={err:.2e}", flush=True)
    assert err <= 1e-4
    assert oracle.error_ratio(D2.cpu().numpy(), At.astype(np.float64).T @ B2.astype(np.float64)) <= 1e-4


def test_strassen_rejects_what_it_cannot_split():
    m = mnn()
    with pytest.raises(m.MnnError) as e:
        m.StrassenGemm(60, 96, 32, 1)          # 60 is not a multiple of 8
    assert e.value.code == -2 or "divisible" in str(e.value)
    with pytest.raises(m.MnnError):
        m.StrassenGemm(64, 96, 31, 1)
    with m.StrassenGemm(64, 96, 32, 1) as sg:
        with pytest.raises(m.MnnError):
            sg.run(torch.zeros(32, 96, device="cuda"), torch.zeros(64, 96, device="cuda"))     # left operand not set


@pytest.mark.parametrize("levels", [1, 2])
def test_pointwise_convolution_through_strassen(levels):
    """The 1x1 scheme with Strassen levels forced: image-strided columns (col -> image, pixel), bias in the
    last combine step."""
    m = mnn()
    layer = ConvLayer("pw_strassen", 4, 64, 14, 14, 96, 1, 1, 1, 0, 1, (0.0, 1.0), BASE_SEED + 9800 + levels)
    x, w, b = draw(layer)
    ref = oracle.conv2d(x, w, b)
    xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
    opt = m.Options(force_kind=m.SCHEME_GEMM1X1, force_variant=levels)
    with m.ConvPlan.for_layer(layer, options=opt) as plan:
        assert plan.scheme.variant == levels and f"levels={levels}" in plan.describe()
        y = torch.full(plan.out_shape, float("nan"), device="cuda")
        plan.run(xd, wd, bd, y)
        plan.run(xd, wd, bd, y)
        torch.cuda.synchronize()
    err = oracle.error_ratio(y.cpu().numpy(), ref)
    assert err <= 1e-4, err


def test_planner_times_strassen_like_any_other_candidate():
    m = mnn()
    m.cache_clear()
    layer = ConvLayer("pw_plan", 16, 256, 14, 14, 512, 1, 1, 1, 0, 1, (0.0, 1.0), BASE_SEED + 9810)
    x, w, b = draw(layer)
    with m.ConvPlan.for_layer(layer) as plan:
        cands = plan.candidates
        assert [(c.kind, c.variant) for c in cands] == [(m.SCHEME_GEMM1X1, v) for v in (0, 1, 2)]
        assert all(c.est_ms > 0 for c in cands)
        chosen = plan.scheme
        best = min(c.est_ms for c in cands)
        assert [c.est_ms for c in cands if c.variant == chosen.variant][0] <= best * 1.02 * (1 + 1e-6)
        y = plan.run(*(torch.from_numpy(a).cuda() for a in (x, w, b)))
        torch.cuda.synchronize()
    assert oracle.error_ratio(y.cpu().numpy(), oracle.conv2d(x, w, b)) <= 1e-4
    m.cache_clear()


@pytest.mark.parametrize("levels", [1, 2])
def test_strassen_at_the_size_of_the_last_pointwise_layer(levels):
    """1024 x 1024 x 784 (cfg4's last layer as one product), the size bench.py times."""
    m = mnn()
    M, R, N = 1024, 1024, 784
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 4040 + levels))
    At = rng.normal(0, np.sqrt(2.0 / R), (R, M)).astype(np.float32)
    B = rng.uniform(0, 1, (R, N)).astype(np.float32)
    ref = At.astype(np.float64).T @ B.astype(np.float64)
    D = torch.full((M, N), float("nan"), device="cuda")
    with m.StrassenGemm(M, N, R, levels) as sg:
        sg.set_left(torch.from_numpy(At).cuda())
        sg.run(torch.from_numpy(B).cuda(), D)
        torch.cuda.synchronize()
    assert oracle.error_ratio(D.cpu().numpy(), ref) <= 1e-4
