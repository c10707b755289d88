"""Parity at the full sizes of the workloads, with the planner's own choice (the launch configuration
bench.py times).  cfg3 and cfg4: the whole output against the oracle.  cfg5: the oracle at 4096 sampled
output coordinates per layer (its full tensor would take minutes of float64 CPU time), drawn over all
images, channels, edges and corners."""
import numpy as np
import pytest
import torch

import oracle
from conv_workloads import config_layers, draw

pytestmark = pytest.mark.gpu


def mnn():
    import paper_2002_12418_amd as m
    return m


def tol_for(scheme, k, m):
    return 1e-3 if (scheme.kind == m.SCHEME_WINOGRAD and scheme.tile_n + k - 1 > 6) else 1e-4


@pytest.mark.parametrize("layer", config_layers(3) + config_layers(4), ids=lambda l: l.name)
def test_cfg3_cfg4_full_tensor(layer):
    m = mnn()
    x, w, b = draw(layer)
    ref = oracle.conv2d(x, w, b, stride=layer.stride, pad=layer.pad, dil=layer.dil)
    xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
    with m.ConvPlan.for_layer(layer) as plan:
        y = torch.full(plan.out_shape, float("nan"), device="cuda")
        plan.run(xd, wd, bd, y)
        torch.cuda.synchronize()
        s = plan.scheme
    got = y.cpu().numpy()
    assert np.isfinite(got).all()
    err = oracle.error_ratio(got, ref)
    print(f"[full] {layer.name} {s.label(layer.k_long)} err={err:.2e}", flush=True)
    assert err <= tol_for(s, layer.k_long, m)


def sample_coords(shape, count, rng):
    N, K, Ho, Wo = shape
    c = np.stack([rng.integers(0, N, count), rng.integers(0, K, count), rng.integers(0, Ho, count), rng.integers(0, Wo, count)], axis=1)
    # force corners, edges and the last tile row/column into the sample
    k = 0
    for n in (0, N - 1):
        for kk in (0, K - 1):
            for oy in (0, 1, Ho // 2, Ho - 2, Ho - 1):
                for ox in (0, 1, Wo // 2, Wo - 2, Wo - 1):
                    c[k] = (n, kk, oy, ox)
                    k += 1
    return c


@pytest.mark.parametrize("layer", config_layers(5), ids=lambda l: l.name)
def test_cfg5_sampled(layer):
    m = mnn()
    x, w, b = draw(layer)
    xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
    rng = np.random.default_rng(layer.seed)
    with m.ConvPlan.for_layer(layer) as plan:
        y = torch.full(plan.out_shape, float("nan"), device="cuda")
        plan.run(xd, wd, bd, y)
        torch.cuda.synchronize()
        s = plan.scheme
        # properties that hold at any size: everything written, finite
        assert bool(torch.isfinite(y).all())
        coords = sample_coords(plan.out_shape, 4096, rng)
    ref = oracle.conv2d_points(x, w, b, coords, stride=layer.stride, pad=layer.pad, dil=layer.dil)
    got = y.cpu().numpy()[coords[:, 0], coords[:, 1], coords[:, 2], coords[:, 3]].astype(np.float64)
    scale = float(torch.max(torch.abs(y)).item())
    err = float(np.max(np.abs(got - ref))) / scale
    print(f"[sampled] {layer.name} {s.label(layer.k_long)} err={err:.2e}", flush=True)
    assert err <= tol_for(s, layer.k_long, m)


def test_operands_of_two_gib_take_the_wide_loader():
    """An input tensor of 2 GiB: past what the GEMM's range-checked 32-bit offsets can address, so the 1x1 and
    the sliding-window schemes must switch to their 64-bit loader.  Oracle at sampled output coordinates."""
    from conv_workloads import ConvLayer, BASE_SEED
    m = mnn()
    n, c, hw, k = 2, 16, 4096, 4
    assert n * c * hw * hw * 4 >= 2**31
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 9900))
    x = rng.random((n, c, hw, hw), dtype=np.float32) * 2 - 1
    xd = torch.from_numpy(x).cuda()
    for name, ksz, stride, pad in (("wide_pw", 1, 1, 0), ("wide_k3s2", 3, 2, 1)):
        layer = ConvLayer(name, n, c, hw, hw, k, ksz, ksz, stride, pad, 1, (-1.0, 1.0), BASE_SEED + 9901)
        w = rng.normal(0, np.sqrt(2.0 / (ksz * ksz * c)), (k, c, ksz, ksz)).astype(np.float32)
        b = rng.uniform(-0.1, 0.1, k).astype(np.float32)
        wd, bd = torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda()
        o = m.Options.defaults()
        o.force_kind = m.SCHEME_GEMM1X1 if ksz == 1 else m.SCHEME_DIRECT
        with m.ConvPlan.for_layer(layer, options=o) as plan:
            y = torch.full(plan.out_shape, float("nan"), device="cuda")
            plan.run(xd, wd, bd, y)
            torch.cuda.synchronize()
            desc = plan.describe()
        coords = sample_coords(layer.out_shape, 2048, np.random.default_rng(5))
        ref = oracle.conv2d_points(x, w, b, coords, stride=stride, pad=pad)
        got = y[coords[:, 0], coords[:, 1], coords[:, 2], coords[:, 3]].cpu().numpy()
        assert np.isfinite(got).all()
        err = float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))
        print(f"[wide] {name} {desc} err={err:.2e}", flush=True)
        assert err <= 1e-4
        assert bool(torch.isfinite(y).all())
        del y


def test_rect_layers_full_tensor():
    """The factorised 7-tap layers bench.py reports (rectangular_kernels), planner's choice, whole output."""
    from conv_workloads import rect_layers
    m = mnn()
    for layer in rect_layers(16):
        x, w, b = draw(layer)
        ref = oracle.conv2d(x, w, b, stride=layer.stride, pad=layer.pad, dil=layer.dil)
        xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
        for opt in (None, m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=2)):
            with m.ConvPlan.for_layer(layer, options=opt) as plan:
                y = torch.full(plan.out_shape, float("nan"), device="cuda")
                plan.run(xd, wd, bd, y)
                torch.cuda.synchronize()
                s, desc = plan.scheme, plan.describe()
            err = oracle.error_ratio(y.cpu().numpy(), ref)
            print(f"[rect] {layer.name} {desc} err={err:.2e}", flush=True)
            assert err <= tol_for(s, layer.k_long, m)
