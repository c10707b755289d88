"""Seeded random layer shapes through every admissible fp32 scheme, against the float64 oracle.

Shapes are drawn to hit what fixed cases miss: channel counts that are not multiples of 4 or 16, planes whose
sizes leave ragged tiles in both directions, one-row / one-column kernels, padding larger and smaller than
'same', strides and dilations, batch sizes that do not divide the GEMM tiles."""
import numpy as np
import pytest
import torch

import oracle
from conv_workloads import BASE_SEED, ConvLayer, draw

pytestmark = pytest.mark.gpu


def mnn():
    import paper_2002_12418_amd as m
    return m


def random_layer(seed):
    rng = np.random.default_rng(4242 + seed)
    kh, kw = [(1, 1), (2, 2), (3, 3), (3, 3), (5, 5), (7, 7), (1, 7), (7, 1), (3, 1), (1, 5), (3, 5), (4, 4)][seed % 12]
    n = int(rng.integers(1, 5))
    c = int(rng.choice([1, 3, 4, 7, 16, 17, 33, 64, 70]))
    k = int(rng.choice([1, 2, 5, 8, 16, 31, 64, 67]))
    h = int(rng.integers(max(kh, 5), 41))
    w = int(rng.integers(max(kw, 5), 41))
    stride = int(rng.choice([1, 1, 1, 2]))
    dil = int(rng.choice([1, 1, 1, 2])) if max(kh, kw) <= 3 else 1
    pad = (int(rng.integers(0, kh // 2 + 2)), int(rng.integers(0, kw // 2 + 2)))
    if (h + 2 * pad[0] - dil * (kh - 1) - 1) < 0 or (w + 2 * pad[1] - dil * (kw - 1) - 1) < 0:
        pad = (kh // 2 * dil, kw // 2 * dil)
    return ConvLayer(f"rand{seed}_{kh}x{kw}", n, c, h, w, k, kh, kw, stride, pad, dil, (-1.0, 1.0), BASE_SEED + 12000 + seed)


@pytest.mark.parametrize("seed", range(48))
def test_random_layer_every_scheme(seed):
    m = mnn()
    layer = random_layer(seed)
    x, w, b = draw(layer, with_bias=(seed % 5 != 0))
    ref = oracle.conv2d(x, w, b, stride=layer.stride, pad=layer.pad, dil=layer.dil)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    bd = torch.from_numpy(b).cuda() if b is not None else None
    schemes = m.enumerate_schemes(layer.n, layer.c_in, layer.h, layer.w, layer.c_out, layer.kh, layer.kw,
                                  stride=layer.stride, pad=layer.pad, dil=layer.dil, options=m.Options(alpha_max=10))
    assert schemes
    for s in schemes:
        print(f"[case] {layer} {s.label(layer.k_long)}", flush=True)
        opt = m.Options(force_kind=s.kind, force_tile_n=s.tile_n, force_prec=s.prec, force_variant=s.variant, alpha_max=10)
        with m.ConvPlan.for_layer(layer, options=opt) as plan:
            y = torch.full(plan.out_shape, float("nan"), device="cuda")
            plan.run(xd, wd, bd, y)
            torch.cuda.synchronize()
        got = y.cpu().numpy()
        assert got.shape == ref.shape and np.isfinite(got).all()
        alpha = s.tile_n + layer.k_long - 1 if s.kind == m.SCHEME_WINOGRAD else 0
        tol = 1e-4 if alpha <= 6 else 1e-3
        err = oracle.error_ratio(got, ref)
        assert err <= tol, (layer, s.label(layer.k_long), err)
    # and whatever the planner picks by timing
    m.cache_clear()
    with m.ConvPlan.for_layer(layer) as plan:
        y = plan.run(xd, wd, bd)
        torch.cuda.synchronize()
        chosen = plan.scheme
    alpha = chosen.tile_n + layer.k_long - 1 if chosen.kind == m.SCHEME_WINOGRAD else 0
    assert oracle.error_ratio(y.cpu().numpy(), ref) <= (1e-4 if alpha <= 6 else 1e-3)
    m.cache_clear()
