"""The matrix-multiplication unit alone (mnn_gemm_f32) against a float64 matrix product, every tile
configuration, ragged shapes, the (col / L, col % L) image mapping of the 1x1 convolution, bias."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def mnn():
    import paper_2002_12418_amd as m
    return m


SHAPES = [
    # M, R, ncols, batch
    (70, 37, 100, 3),
    (130, 50, 260, 2),
    (64, 64, 512, 4),
    (33, 5, 36, 1),
    (256, 130, 392, 2),
]


@pytest.mark.parametrize("shape", SHAPES)
def test_batched_gemm_every_variant(shape):
    m = mnn()
    M, R, P, batch = shape
    rng = np.random.default_rng(sum(shape))
    lda = (M + 3) // 4 * 4
    At = np.zeros((batch, R, lda), np.float32)
    At[:, :, :M] = rng.normal(0, 1, (batch, R, M))
    B = rng.uniform(-1, 1, (batch, R, P)).astype(np.float32)
    ref = np.einsum("brm,brp->bmp", At[:, :, :M].astype(np.float64), B.astype(np.float64))
    Atd, Bd = torch.from_numpy(At).cuda(), torch.from_numpy(B).cuda()
    names = m.gemm_variants()
    for v in range(len(names)):
        print(f"[case] gemm {shape} variant {names[v]}", flush=True)
        D = torch.full((batch, M, P), float("nan"), device="cuda")
        m.gemm_f32(Atd, Bd, D, M=M, ncols=P, R=R, batch=batch, lda=lda, L=P, variant=v,
                   strideA_batch=R * lda, strideB_batch=R * P, strideD_batch=M * P)
        torch.cuda.synchronize()
        got = D.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all(), names[v]
        assert np.max(np.abs(got - ref)) / np.max(np.abs(ref)) < 1e-5, names[v]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("prec,tol", [(2, 3e-5), (1, 1e-2)])
def test_bf16_matrix_core_variants(shape, prec, tol):
    """bf16x3 (hi/lo split, three bf16 MFMAs) keeps about 16 mantissa bits per operand; plain bf16 keeps 8."""
    m = mnn()
    M, R, P, batch = shape
    rng = np.random.default_rng(sum(shape) + prec)
    lda = (M + 3) // 4 * 4
    At = np.zeros((batch, R, lda), np.float32)
    At[:, :, :M] = rng.normal(0, 1, (batch, R, M))
    B = rng.uniform(-1, 1, (batch, R, P)).astype(np.float32)
    ref = np.einsum("brm,brp->bmp", At[:, :, :M].astype(np.float64), B.astype(np.float64))
    Atd, Bd = torch.from_numpy(At).cuda(), torch.from_numpy(B).cuda()
    names = m.gemm_variants(prec)
    assert len(names) > 3
    for v in range(len(names)):
        print(f"[case] gemm prec={prec} {shape} variant {names[v]}", flush=True)
        D = torch.full((batch, M, P), float("nan"), device="cuda")
        m.gemm_f32(Atd, Bd, D, M=M, ncols=P, R=R, batch=batch, lda=lda, L=P, variant=v, prec=prec,
                   strideA_batch=R * lda, strideB_batch=R * P, strideD_batch=M * P)
        torch.cuda.synchronize()
        got = D.cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all(), names[v]
        assert np.max(np.abs(got - ref)) / np.max(np.abs(ref)) < tol, names[v]


def test_bf16_rounding_is_nearest_even():
    """One product per output: with A = identity the kernel returns bf16(B) (plain) or hi + lo (x3) exactly."""
    m = mnn()
    R = M = 16
    P = 64
    rng = np.random.default_rng(5)
    B = rng.normal(0, 1, (1, R, P)).astype(np.float32)
    # exact ties: 1 + 2^-8 rounds to even (1.0), 1 + 3*2^-8 rounds to 1 + 2^-6... in bf16 (8 significant bits)
    B[0, 0, :4] = [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 1.0 + 2.0 ** -8 + 2.0 ** -20]
    At = np.eye(R, dtype=np.float32)[None]
    Atd, Bd = torch.from_numpy(At).cuda(), torch.from_numpy(B).cuda()
    want_bf16 = torch.from_numpy(B).to(torch.bfloat16).to(torch.float32).numpy()      # library RNE conversion
    for prec in (1, 2):
        D = torch.empty((1, M, P), device="cuda")
        m.gemm_f32(Atd, Bd, D, M=M, ncols=P, R=R, batch=1, lda=M, L=P, prec=prec, strideA_batch=R * M,
                   strideB_batch=R * P, strideD_batch=M * P)
        torch.cuda.synchronize()
        got = D.cpu().numpy()
        if prec == 1:
            np.testing.assert_array_equal(got, want_bf16)
        else:
            lo = torch.from_numpy(B - want_bf16).to(torch.bfloat16).to(torch.float32).numpy()
            np.testing.assert_array_equal(got, want_bf16 + lo)
    assert want_bf16[0, 0, 0] == 1.0 and want_bf16[0, 0, 1] == 1.0 + 2.0 ** -6 and want_bf16[0, 0, 3] == 1.0 + 2.0 ** -7


@pytest.mark.parametrize("hw", [49, 36, 7 * 9])
def test_pointwise_mapping_with_bias(hw):
    """Columns are (image, pixel): x[n][c][hw], y[n][k][hw]; hw = 49 forces the unaligned element-wise loads."""
    m = mnn()
    N, C, K = 3, 19, 21
    rng = np.random.default_rng(hw)
    x = rng.uniform(0, 1, (N, C, hw)).astype(np.float32)
    w = rng.normal(0, 1, (K, C)).astype(np.float32)
    b = rng.uniform(-1, 1, (K,)).astype(np.float32)
    ldk = (K + 3) // 4 * 4
    Wt = np.zeros((C, ldk), np.float32)
    Wt[:, :K] = w.T
    ref = np.einsum("kc,ncp->nkp", w.astype(np.float64), x.astype(np.float64)) + b.astype(np.float64)[None, :, None]
    xd, Wtd, bd = (torch.from_numpy(a).cuda() for a in (x, Wt, b))
    names = m.gemm_variants()
    ran = 0
    for v in range(len(names)):
        y = torch.full((N, K, hw), float("nan"), device="cuda")
        m.gemm_f32(Wtd, xd, y, bd, M=K, ncols=N * hw, R=C, batch=1, lda=ldk, L=hw, variant=v,
                   strideB_img=C * hw, strideB_row=hw, strideD_img=K * hw, strideD_row=hw)
        torch.cuda.synchronize()
        got = y.cpu().numpy().astype(np.float64)
        assert np.max(np.abs(got - ref)) / np.max(np.abs(ref)) < 1e-5, names[v]
        ran += 1
    assert ran >= 5


def test_gemm_rejects_bad_descriptors():
    m = mnn()
    a = torch.zeros(64, device="cuda")
    with pytest.raises(m.MnnError):
        m.gemm_f32(a, a, a, M=8, ncols=8, R=8, lda=6)                 # lda not a multiple of 4
    with pytest.raises(m.MnnError):
        m.gemm_f32(a, a, a, M=8, ncols=8, R=8, lda=8, variant=999)
    with pytest.raises(m.MnnError):
        m.gemm_f32(a, a, a, M=0, ncols=8, R=8, lda=8)
