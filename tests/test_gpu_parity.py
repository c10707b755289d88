"""GPU parity: the HIP path through the C ABI against the float64 oracle, element by element.

Tolerances (max|y - ref| / max|ref| over the whole output tensor): 1e-4 for the fp32 direct, GEMM,
F(2,3) and F(4,3) schemes, 1e-3 for larger Winograd tiles.
"""
import numpy as np
import pytest
import torch

import oracle
from conv_workloads import config_layers, draw, selection_table_layers, small_parity_layers

pytestmark = pytest.mark.gpu


def mnn():
    import paper_2002_12418_amd as m
    return m


def tol_for(scheme, k):
    m = mnn()
    if scheme.kind == m.SCHEME_WINOGRAD and scheme.tile_n + k - 1 > 6:
        return 1e-3
    return 1e-4


def forced_options(layer):
    """Every scheme that is admissible for the layer, as (label, Options)."""
    m = mnn()
    out = []
    for s in m.enumerate_schemes(layer.n, layer.c_in, layer.h, layer.w, layer.c_out, layer.kh, layer.kw,
                                 stride=layer.stride, pad=layer.pad, dil=layer.dil):
        out.append((s.label(layer.k_long), m.Options(force_kind=s.kind, force_tile_n=s.tile_n, force_prec=s.prec,
                                                 force_variant=s.variant)))
    return out


def run_and_compare(layer, options, with_bias=True):
    m = mnn()
    x, w, b = draw(layer, with_bias=with_bias)
    ref = oracle.conv2d(x, w, b, stride=layer.stride, pad=layer.pad, dil=layer.dil)
    xd, wd = torch.from_numpy(x).cuda(), torch.from_numpy(w).cuda()
    bd = torch.from_numpy(b).cuda() if b is not None else None
    with m.ConvPlan.for_layer(layer, options=options) as plan:
        y = torch.full(plan.out_shape, float("nan"), dtype=torch.float32, device="cuda")
        plan.run(xd, wd, bd, y)
        torch.cuda.synchronize()
        got = y.cpu().numpy()
        scheme = plan.scheme
    assert got.shape == ref.shape
    assert np.isfinite(got).all(), "output holds NaN/inf or unwritten elements"
    return oracle.error_ratio(got, ref), scheme


@pytest.mark.parametrize("layer", small_parity_layers(), ids=lambda l: l.name)
def test_small_layers_every_scheme(layer):
    for label, opt in forced_options(layer):
        print(f"[case] {layer.name} {label}", flush=True)
        err, scheme = run_and_compare(layer, opt)
        assert err <= tol_for(scheme, layer.k_long), (layer.name, label, err)


@pytest.mark.parametrize("layer", small_parity_layers()[:4], ids=lambda l: l.name)
def test_small_layers_no_bias(layer):
    for label, opt in forced_options(layer):
        print(f"[case] nobias {layer.name} {label}", flush=True)
        err, scheme = run_and_compare(layer, opt, with_bias=False)
        assert err <= tol_for(scheme, layer.k_long), (layer.name, label, err)


@pytest.mark.parametrize("layer", config_layers(1) + config_layers(2), ids=lambda l: l.name)
def test_config1_and_2_every_scheme(layer):
    for label, opt in forced_options(layer):
        print(f"[case] {layer.name} {label}", flush=True)
        err, scheme = run_and_compare(layer, opt)
        assert err <= tol_for(scheme, layer.k_long), (layer.name, label, err)


@pytest.mark.parametrize("layer", config_layers(1) + config_layers(2), ids=lambda l: l.name)
def test_planner_choice_is_correct_and_listed(layer):
    m = mnn()
    m.cache_clear()
    err, scheme = run_and_compare(layer, None)
    assert err <= tol_for(scheme, layer.k_long)
    if layer.stride != 1:
        assert scheme.kind == m.SCHEME_DIRECT


@pytest.mark.parametrize("layer", selection_table_layers(1), ids=lambda l: l.name)
def test_selection_table_settings_every_scheme(layer):
    """The three settings of the paper's scheme-selection comparison (Table 1): 2-tap kernels with 3 and 512
    channels, a 3-tap kernel with 64: every forced scheme and the planner's pick against the oracle."""
    for label, opt in forced_options(layer) + [("planner", None)]:
        print(f"[case] {layer.name} {label}", flush=True)
        err, scheme = run_and_compare(layer, opt)
        assert err <= tol_for(scheme, layer.k_long), (layer.name, label, err)


BF16_TOL = 2e-2        # bound for the bf16-matrix-core variants
BF16X3_TOL = 5e-4      # what the split-operand variant is held to here (measured <= 3.1e-4 at alpha = 8)


@pytest.mark.parametrize("layer", small_parity_layers() + config_layers(1) + config_layers(2), ids=lambda l: l.name)
def test_bf16_matrix_core_schemes(layer):
    """Every scheme the planner may use with allow_bf16: bf16x3 for all GEMM-stage schemes, plain bf16 for the
    1x1 and sliding-window schemes."""
    m = mnn()
    seen = 0
    for s in m.enumerate_schemes(layer.n, layer.c_in, layer.h, layer.w, layer.c_out, layer.kh, layer.kw,
                                 stride=layer.stride, pad=layer.pad, dil=layer.dil, options=m.Options(allow_bf16=1)):
        if s.prec == m.GEMM_FP32:
            continue
        print(f"[case] {layer.name} {s.label(layer.k_long)}", flush=True)
        opt = m.Options(force_kind=s.kind, force_tile_n=s.tile_n, force_prec=s.prec, force_variant=s.variant)
        err, scheme = run_and_compare(layer, opt)
        assert scheme.prec == s.prec
        # split operands: this library's own 5e-4 up to alpha = 8; alpha = 9 and 10 measure about 1e-3 and are held to the bf16 bound
        tight = s.prec == m.GEMM_BF16X3 and not (s.kind == m.SCHEME_WINOGRAD and s.tile_n + layer.k_long - 1 > 8)
        assert err <= (BF16X3_TOL if tight else BF16_TOL), (layer.name, s.label(layer.k_long), err)
        seen += 1
    assert seen >= 2


def test_planner_with_bf16_allowed_stays_within_the_bf16_bound():
    m = mnn()
    m.cache_clear()
    for layer in config_layers(2)[:5]:
        err, scheme = run_and_compare(layer, m.Options(allow_bf16=1))
        assert err <= (tol_for(scheme, layer.k_long) if scheme.prec == m.GEMM_FP32 else BF16_TOL)
    m.cache_clear()
