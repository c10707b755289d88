"""mnn_conv_run_static -- the entry point that allocates no device memory -- against mnn_conv_plan + mnn_conv_run
with the same forced scheme (and against the float64 oracle), through the C ABI.  Calls come in pairs on one
stream, the second with a smaller input than the first: the fixed scratch array keeps the first call's contents,
and nothing of them may leak into the second result."""
import numpy as np
import pytest
import torch

import oracle
from conv_workloads import BASE_SEED, ConvLayer, draw

pytestmark = pytest.mark.gpu


def mnn():
    import paper_2002_12418_amd as m
    return m


def L(i, n, c, h, w, k, kh, kw, s=1, p=0, d=1):
    return ConvLayer(f"static{i}", n, c, h, w, k, kh, kw, s, p, d, (-1.0, 1.0), BASE_SEED + 9600 + i)


# (first layer, second and smaller layer, tile_n)
PAIRS = [
    (L(0, 3, 37, 30, 27, 50, 3, 3, 1, 1), L(1, 1, 9, 11, 10, 6, 3, 3, 1, 1), 4),      # F(4,3), ragged tiles, K % 4 != 0
    (L(2, 2, 24, 21, 33, 17, 3, 3, 1, 1), L(3, 1, 5, 8, 9, 3, 3, 3, 1, 0), 2),        # F(2,3)
    (L(4, 2, 16, 26, 26, 20, 5, 5, 1, 2), L(5, 1, 4, 12, 13, 7, 5, 5, 1, 2), 4),      # F(4,5), alpha = 8
    (L(6, 2, 12, 19, 23, 10, 1, 7, 1, (0, 3)), L(7, 1, 3, 9, 14, 5, 7, 1, 1, (3, 0)), 2),   # kernels with one row / column
    (L(8, 4, 30, 29, 29, 45, 3, 3, 2, 1), L(9, 1, 7, 13, 12, 9, 3, 3, 1, 2, 2), 0),   # sliding window: stride 2, dilation 2
    (L(10, 3, 70, 14, 14, 130, 1, 1), L(11, 2, 19, 7, 7, 21, 1, 1), 0),               # 1x1 GEMM
]


@pytest.mark.parametrize("first,second,tile_n", PAIRS, ids=lambda v: v.name if hasattr(v, "name") else f"n{v}")
def test_static_entry_point_matches_planned_run(first, second, tile_n):
    m = mnn()
    for layer in (first, second):
        x, w, b = draw(layer)
        ref = oracle.conv2d(x, w, b, stride=layer.stride, pad=layer.pad, dil=layer.dil)
        xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
        y_static = torch.full(layer.out_shape, float("nan"), device="cuda")
        print(f"[case] static {layer.name} tile_n={tile_n}", flush=True)
        m.conv_run_static(layer, tile_n, xd, wd, bd, y_static)
        if tile_n:
            opt = m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=tile_n, force_variant=m.WINO_UNFUSED)
        else:
            opt = m.Options(force_kind=m.SCHEME_GEMM1X1 if layer.kh == 1 and layer.kw == 1 else m.SCHEME_DIRECT)
        with m.ConvPlan.for_layer(layer, options=opt) as plan:
            y_plan = plan.run(xd, wd, bd)
            torch.cuda.synchronize()
        got, want = y_static.cpu().numpy(), y_plan.cpu().numpy()
        assert np.isfinite(got).all()
        alpha = tile_n + layer.k_long - 1 if tile_n else 0
        tol = 1e-3 if alpha > 6 else 1e-4
        # same kernels, possibly another GEMM tile configuration (the plan times them, the static call does not)
        assert oracle.error_ratio(got, want) <= tol
        assert oracle.error_ratio(got, ref) <= tol
        # no bias
        y2 = torch.full(layer.out_shape, float("nan"), device="cuda")
        m.conv_run_static(layer, tile_n, xd, wd, None, y2)
        torch.cuda.synchronize()
        assert oracle.error_ratio(y2.cpu().numpy(), oracle.conv2d(x, w, None, stride=layer.stride, pad=layer.pad, dil=layer.dil)) <= tol


def test_static_entry_point_rejects_what_does_not_fit():
    m = mnn()
    assert m.static_scratch_bytes() == 64 << 20
    big = L(20, 16, 256, 128, 128, 256, 3, 3, 1, 1)          # V and M of hundreds of MB
    t = torch.zeros(16, device="cuda")
    with pytest.raises(m.MnnError) as e:
        m.conv_run_static(big, 4, t, t, None, t)
    assert e.value.code == -2 and "static buffer holds" in str(e.value)
    with pytest.raises(m.MnnError) as e:
        m.conv_run_static(L(21, 1, 4, 9, 9, 4, 3, 3, 2, 1), 2, t, t, None, t)      # Winograd on a strided layer
    assert e.value.code == -2
    with pytest.raises(m.MnnError) as e:
        m.conv_run_static(L(22, 1, 4, 9, 9, 4, 3, 3, 1, 1), -1, t, t, None, t)
    assert e.value.code == -1
