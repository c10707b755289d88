"""Each Winograd stage on its own against the float64 step-by-step oracle: U = G w G^T, V = B^T d B,
M = U V (unfused arrangement), in the library's row layouts and in the blocked layouts of the fused
arrangement."""
import numpy as np
import pytest
import torch

import oracle
from oracle import winograd
from conv_workloads import ConvLayer, draw, BASE_SEED

pytestmark = pytest.mark.gpu


def mnn():
    import paper_2002_12418_amd as m
    return m


CASES = [
    # n, k, N, C, H, W, K, pad
    (2, 3, 2, 5, 9, 7, 6, 1),
    (4, 3, 3, 17, 14, 9, 33, 1),
    (6, 3, 1, 8, 20, 20, 8, 1),
    (4, 5, 1, 6, 12, 16, 7, 2),
    (2, 7, 1, 4, 16, 16, 5, 3),
    (3, 2, 2, 6, 9, 9, 4, 0),
    # more than 1024 tiles: the tiled layout [channel][64 tiles][position][tile in block], last block ragged
    (4, 3, 5, 6, 60, 62, 7, 1),
    (6, 3, 3, 5, 111, 120, 4, 1),
]


def relerr(got, ref):
    return float(np.max(np.abs(got.astype(np.float64) - ref)) / max(np.max(np.abs(ref)), 1e-30))


@pytest.mark.parametrize("case", CASES)
def test_unfused_stage_buffers(case):
    m = mnn()
    n, k, N, C, H, W, K, pad = case
    layer = ConvLayer("t", N, C, H, W, K, k, k, 1, pad, 1, (-1.0, 1.0), BASE_SEED + 500 + sum(case))
    x, w, b = draw(layer)
    yref, st = winograd.winograd_conv2d(x, w, b, n, pad=pad, return_stages=True)
    a = n + k - 1
    xd, wd, bd = (torch.from_numpy(t).cuda() for t in (x, w, b))
    opt = m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=n, force_variant=m.WINO_UNFUSED)
    with m.ConvPlan.for_layer(layer, options=opt) as plan:
        info = plan.info
        y = plan.run(xd, wd, bd)
        torch.cuda.synchronize()
        P, ldp, ldk = info["p"], info["ldp"], info["ldk"]
        assert P == st["V"].shape[-1] and info["alpha"] == a
        U = plan.buffer_to_numpy(m.BUF_U).reshape(a * a, C, ldk)
        V, M = plan.buffer_to_numpy(m.BUF_V), plan.buffer_to_numpy(m.BUF_M)
        assert bool(info["tiled"]) == (P >= 1024)
        if info["tiled"]:
            pb = info["pb"]
            assert pb == (P + 63) // 64 and ldp == 64 * pb
            V = V.reshape(C, pb, a * a, 64).transpose(2, 0, 1, 3).reshape(a * a, C, ldp)
            M = M.reshape(K, pb, a * a, 64).transpose(2, 0, 1, 3).reshape(a * a, K, ldp)
        else:
            V, M = V.reshape(a * a, C, ldp), M.reshape(a * a, K, ldp)
    Uref = st["U"].reshape(a * a, K, C).transpose(0, 2, 1)            # library keeps U transposed: [xi][c][k]
    assert relerr(U[:, :, :K], Uref) < 1e-5
    assert np.all(U[:, :, K:] == 0)
    assert relerr(V[:, :, :P], st["V"].reshape(a * a, C, P)) < 1e-5
    assert np.all(V[:, :, P:] == 0)
    assert relerr(M[:, :, :P], st["M"].reshape(a * a, K, P)) < 1e-4
    assert oracle.error_ratio(y.cpu().numpy(), yref) < 1e-4


@pytest.mark.parametrize("case", CASES[:4])
def test_blocked_stage_buffers(case):
    """Fused arrangement: Ub[b][c/4][a][k/16][c%4][k%16] and Vb[b][c/4][a][p/16][c%4][p%16], zero padding."""
    m = mnn()
    n, k, N, C, H, W, K, pad = case
    layer = ConvLayer("t", N, C, H, W, K, k, k, 1, pad, 1, (-1.0, 1.0), BASE_SEED + 500 + sum(case))
    x, w, b = draw(layer)
    yref, st = winograd.winograd_conv2d(x, w, b, n, pad=pad, return_stages=True)
    a = n + k - 1
    xd, wd, bd = (torch.from_numpy(t).cuda() for t in (x, w, b))
    opt = m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=n, force_variant=m.WINO_FUSED_OUT_32)
    with m.ConvPlan.for_layer(layer, options=opt) as plan:
        info = plan.info
        y = plan.run(xd, wd, bd)
        torch.cuda.synchronize()
        P, kg, pg = info["p"], info["kg"], info["pg"]
        U = plan.buffer_to_numpy(m.BUF_U)
        V = plan.buffer_to_numpy(m.BUF_V)
        assert plan.buffer(m.BUF_M)[0] == 0                           # the product tensor is never materialised
    cch = U.size // (a * a * kg * 64)
    assert cch * 4 >= C and V.size == a * cch * a * pg * 64
    Ub = U.reshape(a, cch, a, kg, 4, 16)                              # [b][cc][a][kgroup][c%4][k%16]
    Vb = V.reshape(a, cch, a, pg, 4, 16)
    Ufull = Ub.transpose(2, 0, 1, 4, 3, 5).reshape(a, a, cch * 4, kg * 16)   # [a][b][c][k]
    Vfull = Vb.transpose(2, 0, 1, 4, 3, 5).reshape(a, a, cch * 4, pg * 16)   # [a][b][c][p]
    assert relerr(Ufull[:, :, :C, :K], st["U"].transpose(0, 1, 3, 2)) < 1e-5
    assert relerr(Vfull[:, :, :C, :P], st["V"]) < 1e-5
    for full, lim in ((Ufull, (C, K)), (Vfull, (C, P))):
        assert np.all(full[:, :, lim[0]:, :] == 0) and np.all(full[:, :, :, lim[1]:] == 0)
    assert oracle.error_ratio(y.cpu().numpy(), yref) < 1e-4


RECT_CASES = [
    # n, kh, kw, N, C, H, W, K, pad
    (2, 1, 7, 1, 5, 9, 20, 6, (0, 3)),
    (2, 7, 1, 2, 6, 17, 13, 9, (3, 0)),
    (4, 1, 3, 2, 10, 9, 22, 5, (0, 1)),
    (6, 3, 1, 1, 7, 20, 5, 4, (1, 0)),
    (4, 5, 1, 1, 3, 23, 6, 4, (0, 0)),
    # several taps on both axes
    (2, 3, 5, 1, 4, 10, 12, 3, (1, 2)),
    (4, 5, 2, 2, 7, 14, 9, 6, (0, 0)),
    (2, 2, 7, 1, 5, 11, 19, 9, (1, 2)),
    (5, 4, 3, 2, 9, 13, 15, 10, (2, 1)),
]


@pytest.mark.parametrize("case", RECT_CASES)
def test_single_row_or_column_stage_buffers(case):
    """Kernels that are not square: U, V, M hold alpha_h x alpha_w positions (one of the two equal to 1 for kernels with
    one row or column)."""
    m = mnn()
    n, kh, kw, N, C, H, W, K, pad = case
    layer = ConvLayer("t", N, C, H, W, K, kh, kw, 1, pad, 1, (-1.0, 1.0), BASE_SEED + 600 + n + 7 * kh + kw)
    x, w, b = draw(layer)
    yref, st = winograd.winograd_conv2d(x, w, b, n, pad=pad, return_stages=True)
    ah, aw = st["U"].shape[:2]
    xd, wd, bd = (torch.from_numpy(t).cuda() for t in (x, w, b))
    opt = m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=n, force_variant=m.WINO_UNFUSED)
    with m.ConvPlan.for_layer(layer, options=opt) as plan:
        info = plan.info
        assert (info["alpha"], info["alpha_w"]) == (ah, aw)
        assert (info["tile_n"], info["tile_n_w"]) == (1 if kh == 1 else n, 1 if kw == 1 else n)
        y = plan.run(xd, wd, bd)
        torch.cuda.synchronize()
        P, ldp, ldk = info["p"], info["ldp"], info["ldk"]
        assert P == st["V"].shape[-1]
        U = plan.buffer_to_numpy(m.BUF_U).reshape(ah * aw, C, ldk)
        V = plan.buffer_to_numpy(m.BUF_V).reshape(ah * aw, C, ldp)
        M = plan.buffer_to_numpy(m.BUF_M).reshape(ah * aw, K, ldp)
        assert "x" in plan.describe()
    assert relerr(U[:, :, :K], st["U"].reshape(ah * aw, K, C).transpose(0, 2, 1)) < 1e-5
    assert relerr(V[:, :, :P], st["V"].reshape(ah * aw, C, P)) < 1e-5
    assert relerr(M[:, :, :P], st["M"].reshape(ah * aw, K, P)) < 1e-4
    assert oracle.error_ratio(y.cpu().numpy(), oracle.conv2d(x, w, b, pad=pad)) < (1e-3 if max(ah, aw) > 6 else 1e-4)
