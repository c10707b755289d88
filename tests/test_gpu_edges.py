"""Edge cases through the C ABI: guard bands around the output, unaligned tensor bases, batch 1,
one channel, pad 0, outputs smaller than one tile, alpha up to 12, point scale f."""
import numpy as np
import pytest
import torch

import oracle
from conv_workloads import ConvLayer, draw, BASE_SEED

pytestmark = pytest.mark.gpu


def mnn():
    import paper_2002_12418_amd as m
    return m


def all_forced(m, layer, **kw):
    out = []
    for s in m.enumerate_schemes(layer.n, layer.c_in, layer.h, layer.w, layer.c_out, layer.kh, layer.kw,
                                 stride=layer.stride, pad=layer.pad, dil=layer.dil, options=m.Options(**kw) if kw else None):
        out.append((s, m.Options(force_kind=s.kind, force_tile_n=s.tile_n, force_prec=s.prec, force_variant=s.variant, **kw)))
    return out


def tol_for(s, k, m):
    return 1e-3 if (s.kind == m.SCHEME_WINOGRAD and s.tile_n + k - 1 > 6) else 1e-4


LAYERS = [
    ConvLayer("one_tile", 1, 3, 4, 4, 5, 3, 3, 1, 1, 1, (-1.0, 1.0), BASE_SEED + 801),
    ConvLayer("single_channel", 2, 1, 10, 11, 1, 3, 3, 1, 1, 1, (-1.0, 1.0), BASE_SEED + 802),
    ConvLayer("odd_everything", 3, 7, 13, 17, 19, 3, 3, 1, 0, 1, (-1.0, 1.0), BASE_SEED + 803),
    ConvLayer("pw_odd", 2, 5, 7, 7, 9, 1, 1, 1, 0, 1, (0.0, 1.0), BASE_SEED + 804),
    ConvLayer("k2", 1, 6, 12, 12, 10, 2, 2, 1, 0, 1, (-1.0, 1.0), BASE_SEED + 805),
    ConvLayer("s2d2", 2, 6, 15, 14, 10, 3, 3, 2, 2, 2, (-1.0, 1.0), BASE_SEED + 806),
]


@pytest.mark.parametrize("layer", LAYERS, ids=lambda l: l.name)
@pytest.mark.parametrize("shift", [0, 1])
def test_guard_bands_and_unaligned_bases(layer, shift):
    """Output sits inside a larger buffer filled with a canary; shift = 1 also makes every tensor base
    4-byte instead of 16-byte aligned, which must take the element-wise paths."""
    m = mnn()
    x, w, b = draw(layer)
    ref = oracle.conv2d(x, w, b, stride=layer.stride, pad=layer.pad, dil=layer.dil)
    guard = 64 + shift

    def place(a):
        buf = torch.full((a.size + 2 * guard,), 777.0, device="cuda")
        view = buf[guard:guard + a.size].view(a.shape)
        view.copy_(torch.from_numpy(a))
        return buf, view

    (_, xd), (_, wd), (_, bd) = place(x), place(w), place(b)
    for s, opt in all_forced(m, layer):
        print(f"[case] {layer.name} shift={shift} {s.label(layer.k_long)}", flush=True)
        ybuf = torch.full((ref.size + 2 * guard,), 777.0, device="cuda")
        y = ybuf[guard:guard + ref.size].view(ref.shape)
        with m.ConvPlan.for_layer(layer, options=opt) as plan:
            plan.run(xd, wd, bd, y)
            torch.cuda.synchronize()
        host = ybuf.cpu().numpy()
        assert np.all(host[:guard] == 777.0) and np.all(host[guard + ref.size:] == 777.0), "wrote outside the output"
        assert oracle.error_ratio(host[guard:guard + ref.size].reshape(ref.shape), ref) <= tol_for(s, layer.k_long, m)


def test_large_alpha_and_point_scale():
    """alpha up to 10 (F(6,5)) runs through the unfused arrangement within 1e-3; f = 1 is less accurate than 1/2;
    alpha_max above 10 is refused because the fp32 error of such tiles is above 1e-2."""
    m = mnn()
    layer = ConvLayer("k5", 1, 6, 24, 24, 8, 5, 5, 1, 2, 1, (-1.0, 1.0), BASE_SEED + 810)
    x, w, b = draw(layer)
    ref = oracle.conv2d(x, w, b, pad=2)
    xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
    errs = {}
    for n, f in ((6, 0.5), (5, 0.5), (4, 0.5), (4, 1.0)):
        opt = m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=n, force_variant=0, alpha_max=10, point_scale_f=f)
        with m.ConvPlan.for_layer(layer, options=opt) as plan:
            y = plan.run(xd, wd, bd)
            torch.cuda.synchronize()
            errs[(n, f)] = oracle.error_ratio(y.cpu().numpy(), ref)
    print(errs, flush=True)
    assert errs[(4, 0.5)] <= 1e-3 and errs[(5, 0.5)] <= 1e-3 and errs[(6, 0.5)] <= 1e-3
    assert errs[(4, 0.5)] < errs[(4, 1.0)]
    with pytest.raises(m.MnnError) as e:
        m.ConvPlan.for_layer(layer, options=m.Options(alpha_max=12))
    assert e.value.code == -2


def test_runs_are_bit_reproducible():
    m = mnn()
    layer = ConvLayer("repro", 2, 24, 20, 20, 40, 3, 3, 1, 1, 1, (-1.0, 1.0), BASE_SEED + 811)
    x, w, b = draw(layer)
    xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
    for s, opt in all_forced(m, layer):
        with m.ConvPlan.for_layer(layer, options=opt) as plan:
            y1 = plan.run(xd, wd, bd).clone()
            y2 = plan.run(xd, wd, bd)
            torch.cuda.synchronize()
            assert torch.equal(y1, y2), s.label(3)


def test_point_scale_per_alpha_lowers_the_error_of_the_largest_tiles():
    """alpha = 10 (F(8,3), F(4,7)): the paper's f = 0.5 gives 1e-4 .. 4e-4, points spaced 0.425 apart (what
    point_scale_f = 0 selects for alpha >= 9) several times less; for alpha <= 8 the two settings are the same."""
    m = mnn()
    for n, k, c in ((8, 3, 96), (4, 7, 64)):
        layer = ConvLayer(f"ps_F{n}{k}", 2, c, 33, 29, 24, k, k, 1, k // 2, 1, (-1.0, 1.0), BASE_SEED + 9600 + n + k)
        x, w, b = draw(layer)
        ref = oracle.conv2d(x, w, b, pad=k // 2)
        xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
        errs = {}
        for f in (0.5, 0.0):
            o = m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=n, force_variant=m.WINO_UNFUSED, alpha_max=10, point_scale_f=f)
            with m.ConvPlan.for_layer(layer, options=o) as plan:
                y = plan.run(xd, wd, bd)
                torch.cuda.synchronize()
            errs[f] = oracle.error_ratio(y.cpu().numpy(), ref)
        print(f"[point scale] F({n},{k}) C={c}: f=0.5 {errs[0.5]:.2e}, per-alpha {errs[0.0]:.2e}", flush=True)
        assert errs[0.0] <= 3e-4 and errs[0.5] <= 1e-3
        assert errs[0.0] < 0.7 * errs[0.5]
    layer = ConvLayer("ps_F63", 1, 32, 20, 20, 16, 3, 3, 1, 1, 1, (-1.0, 1.0), BASE_SEED + 9650)
    x, w, b = draw(layer)
    xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
    outs = []
    for f in (0.5, 0.0):
        o = m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=6, force_variant=m.WINO_UNFUSED, point_scale_f=f)
        with m.ConvPlan.for_layer(layer, options=o) as plan:
            outs.append(plan.run(xd, wd, bd).clone())
    torch.cuda.synchronize()
    assert torch.equal(outs[0], outs[1])


DEGENERATE = [
    ConvLayer("all_ones", 1, 1, 1, 1, 1, 1, 1, 1, 0, 1, (-1.0, 1.0), BASE_SEED + 851),              # a single multiply-add
    ConvLayer("output_1x1", 2, 5, 3, 3, 4, 3, 3, 1, 0, 1, (-1.0, 1.0), BASE_SEED + 852),             # kernel = image
    ConvLayer("one_row", 2, 6, 1, 37, 5, 1, 3, 1, (0, 1), 1, (-1.0, 1.0), BASE_SEED + 853),           # H = 1, 1x3 kernel
    ConvLayer("one_column", 1, 4, 29, 1, 7, 5, 1, 1, (2, 0), 1, (-1.0, 1.0), BASE_SEED + 854),        # W = 1, 5x1 kernel
    ConvLayer("deep_tiny", 1, 2048, 4, 4, 8, 3, 3, 1, 1, 1, (-1.0, 1.0), BASE_SEED + 855),            # long reduction, 16 outputs per channel
    ConvLayer("wide_out_tiny", 1, 3, 5, 5, 1500, 3, 3, 1, 1, 1, (-1.0, 1.0), BASE_SEED + 856),        # many output channels
    ConvLayer("many_images", 300, 3, 5, 5, 5, 3, 3, 1, 1, 1, (-1.0, 1.0), BASE_SEED + 857),           # batch much larger than the image
    ConvLayer("pad_only_border", 1, 3, 2, 2, 3, 3, 3, 1, 2, 1, (-1.0, 1.0), BASE_SEED + 858),         # most taps fall on padding
    ConvLayer("stride_beyond_image", 2, 4, 9, 9, 3, 3, 3, 7, 1, 1, (-1.0, 1.0), BASE_SEED + 859),     # stride larger than the kernel
    ConvLayer("k9_direct", 1, 3, 20, 20, 4, 9, 9, 1, 4, 1, (-1.0, 1.0), BASE_SEED + 860),             # more taps than the Winograd path takes
    ConvLayer("pw_one_pixel", 7, 33, 1, 1, 65, 1, 1, 1, 0, 1, (0.0, 1.0), BASE_SEED + 861),           # 1x1 kernel on 1x1 images
]


@pytest.mark.parametrize("layer", DEGENERATE, ids=lambda l: l.name)
def test_degenerate_shapes_every_scheme(layer):
    """Shapes at the ends of the ranges: one element, one row or column, output 1 x 1, reductions and channel counts far
    larger than the image, a batch far larger than the image, taps mostly on padding; every admissible scheme and the
    planner's own choice against the oracle."""
    m = mnn()
    x, w, b = draw(layer)
    ref = oracle.conv2d(x, w, b, stride=layer.stride, pad=layer.pad, dil=layer.dil)
    xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
    cases = all_forced(m, layer) + [(None, None)]
    assert len(cases) >= 2
    for s, opt in cases:
        print(f"[case] {layer.name} {s.label(layer.k_long) if s else 'planner'}", flush=True)
        m.cache_clear()
        with m.ConvPlan.for_layer(layer, options=opt) as plan:
            y = torch.full(plan.out_shape, float("nan"), dtype=torch.float32, device="cuda")
            plan.run(xd, wd, bd, y)
            torch.cuda.synchronize()
            chosen = plan.scheme
        got = y.cpu().numpy()
        assert got.shape == ref.shape and np.isfinite(got).all()
        assert oracle.error_ratio(got, ref) <= tol_for(chosen, layer.k_long, m), (layer.name, chosen.label(layer.k_long))


def test_fused_64x64_with_a_tail_of_32x32_workgroups():
    """50176 tiles and 64 output channels make 784 workgroups of 64 x 64, one and a half times what the device holds:
    the library gives the 64 x 64 kernel the blocks of the full round and the rest of the tiles to 32 x 32 workgroups.
    Whole tensor against the oracle, and the same bits as the 32 x 32 arrangement alone (same order of additions)."""
    m = mnn()
    layer = ConvLayer("split_tail", 16, 8, 112, 112, 64, 3, 3, 1, 1, 1, (-1.0, 1.0), BASE_SEED + 870)
    x, w, b = draw(layer)
    ref = oracle.conv2d(x, w, b, stride=1, pad=1)
    xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
    outs = {}
    for variant in (m.WINO_FUSED_OUT_64, m.WINO_FUSED_OUT_32):
        opt = m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=2, force_variant=variant)
        with m.ConvPlan.for_layer(layer, options=opt) as plan:
            y = torch.full(plan.out_shape, float("nan"), dtype=torch.float32, device="cuda")
            plan.run(xd, wd, bd, y)
            torch.cuda.synchronize()
        assert oracle.error_ratio(y.cpu().numpy(), ref) <= 1e-4
        outs[variant] = y
    assert torch.equal(outs[m.WINO_FUSED_OUT_64], outs[m.WINO_FUSED_OUT_32])


@pytest.mark.parametrize("case", [
    # name, N, C, H, W, K, k, pad, n
    ("f47_ragged", 2, 13, 37, 41, 70, 7, 3, 4),          # channels, output channels and tiles all ragged
    ("f46_ragged", 1, 9, 30, 26, 33, 6, 2, 4),
    ("f47_tail", 3, 4, 320, 320, 64, 7, 3, 4),           # 300 blocks of 64 tiles: 256 as 64 x 64, 44 as 32 x 32 workgroups
], ids=lambda c: c[0])
def test_fused_64x64_as_sixteen_one_tile_wavefronts(case):
    """F(4,6) and F(4,7) do not fit two 16 x 16 tiles per wavefront; their 64 x 64 blocks are sixteen wavefronts of one
    tile each.  Whole tensor against the oracle, and the same bits as the 32 x 32 arrangement."""
    m = mnn()
    name, N, C, H, W, K, k, pad, n = case
    layer = ConvLayer(name, N, C, H, W, K, k, k, 1, pad, 1, (-1.0, 1.0), BASE_SEED + 880 + k + C)
    x, w, b = draw(layer)
    ref = oracle.conv2d(x, w, b, stride=1, pad=pad)
    xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
    outs = {}
    for variant in (m.WINO_FUSED_OUT_64, m.WINO_FUSED_OUT_32):
        opt = m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=n, force_variant=variant)
        with m.ConvPlan.for_layer(layer, options=opt) as plan:
            assert plan.scheme.variant == variant
            y = torch.full(plan.out_shape, float("nan"), dtype=torch.float32, device="cuda")
            plan.run(xd, wd, bd, y)
            torch.cuda.synchronize()
        assert oracle.error_ratio(y.cpu().numpy(), ref) <= 1e-3
        outs[variant] = y
    assert torch.equal(outs[m.WINO_FUSED_OUT_64], outs[m.WINO_FUSED_OUT_32])


def test_weights_rewritten_behind_the_same_pointer_are_prepared_again():
    """The prepared weights (G w G^T, the transposed weights of the other schemes) are cached per weight pointer.
    New values behind an unchanged pointer -- an in-place update, a rewrite torch does not count -- must not be served
    from the old preparation: the binding notices torch's version counter, mnn_conv_set_weights is the explicit call."""
    m = mnn()
    layer = ConvLayer("rewrite", 2, 12, 14, 13, 10, 3, 3, 1, 1, 1, (-1.0, 1.0), BASE_SEED + 830)
    x, w, b = draw(layer)
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 831))
    w2 = rng.normal(0.0, 0.2, w.shape).astype(np.float32)
    w3 = rng.normal(0.0, 0.2, w.shape).astype(np.float32)
    refs = [oracle.conv2d(x, ww, b, pad=1) for ww in (w, w2, w3)]
    xd, bd = torch.from_numpy(x).cuda(), torch.from_numpy(b).cuda()
    for s, opt in all_forced(m, layer):
        print(f"[case] rewrite {s.label(3)}", flush=True)
        wd = torch.from_numpy(w).cuda()
        with m.ConvPlan.for_layer(layer, options=opt) as plan:
            y = plan.run(xd, wd, bd)
            assert oracle.error_ratio(y.cpu().numpy(), refs[0]) <= tol_for(s, 3, m)
            wd.copy_(torch.from_numpy(w2))                      # in place: same address, torch's counter moves
            y = plan.run(xd, wd, bd)
            assert oracle.error_ratio(y.cpu().numpy(), refs[1]) <= tol_for(s, 3, m), "stale prepared weights were used"
            # a write that torch's counter of this tensor does not see (.data has a counter of its own), then the explicit call
            wd.data.copy_(torch.from_numpy(w3))
            plan.set_weights(wd)
            y = plan.run(xd, wd, bd)
            assert oracle.error_ratio(y.cpu().numpy(), refs[2]) <= tol_for(s, 3, m)
