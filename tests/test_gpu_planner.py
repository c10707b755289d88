"""Pre-inference planner on the device: the choice is one of the candidates and within 2 % of the fastest
one measured, it is cached per shape, forced schemes are honoured, and a plan can be re-run with new
weights."""
import numpy as np
import pytest
import torch

import oracle
from conv_workloads import config_layers, draw

pytestmark = pytest.mark.gpu


def mnn():
    import paper_2002_12418_amd as m
    return m


@pytest.mark.parametrize("layer", [config_layers(1)[0], config_layers(2)[1], config_layers(2)[5], config_layers(4)[3].with_batch(2)],
                         ids=lambda l: l.name)
def test_choice_is_the_measured_best_and_is_cached(layer):
    m = mnn()
    m.cache_clear()
    assert m.cache_size() == 0
    with m.ConvPlan.for_layer(layer) as plan:
        chosen, cands = plan.scheme, plan.candidates
    listed = m.enumerate_schemes(layer.n, layer.c_in, layer.h, layer.w, layer.c_out, layer.kh, layer.kw,
                                 stride=layer.stride, pad=layer.pad, dil=layer.dil)
    assert [(c.kind, c.tile_n, c.variant) for c in cands] == [(c.kind, c.tile_n, c.variant) for c in listed]
    assert any((c.kind, c.tile_n, c.prec, c.variant) == (chosen.kind, chosen.tile_n, chosen.prec, chosen.variant) for c in cands)
    timed = [c for c in cands if c.est_ms >= 0]
    if len(cands) > 1:
        assert len(timed) == len(cands)
        best = min(c.est_ms for c in timed)
        mine = [c for c in timed if (c.kind, c.tile_n, c.variant) == (chosen.kind, chosen.tile_n, chosen.variant)][0]
        assert mine.est_ms <= best * 1.02 * (1 + 1e-6)
    if layer.kh == 1:
        assert chosen.kind == m.SCHEME_GEMM1X1
    if layer.stride != 1:
        assert chosen.kind == m.SCHEME_DIRECT
    assert m.cache_size() == 1
    # second plan for the same shape: served from the cache, nothing is timed again
    with m.ConvPlan.for_layer(layer) as plan2:
        again = plan2.scheme
        assert all(c.est_ms < 0 for c in plan2.candidates) or len(plan2.candidates) == 1
    assert (again.kind, again.tile_n, again.prec, again.variant) == (chosen.kind, chosen.tile_n, chosen.prec, chosen.variant)
    assert m.cache_size() == 1
    # a different batch size is a different key
    with m.ConvPlan.for_layer(layer.with_batch(layer.n + 1)):
        pass
    assert m.cache_size() == 2
    m.cache_clear()


def test_forced_scheme_and_weight_refresh():
    m = mnn()
    layer = config_layers(1)[0]
    x, w, b = draw(layer)
    w2 = (w * 0.5 + 0.01).astype(np.float32)
    xd, wd, bd, w2d = (torch.from_numpy(a).cuda() for a in (x, w, b, w2))
    ref1 = oracle.conv2d(x, w, b, pad=1)
    ref2 = oracle.conv2d(x, w2, b, pad=1)
    opt = m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=4, force_variant=m.WINO_UNFUSED)
    with m.ConvPlan.for_layer(layer, options=opt) as plan:
        s = plan.scheme
        assert (s.kind, s.tile_n, s.variant) == (m.SCHEME_WINOGRAD, 4, m.WINO_UNFUSED)
        assert plan.workspace_bytes > 0
        y = plan.run(xd, wd, bd)
        torch.cuda.synchronize()
        assert oracle.error_ratio(y.cpu().numpy(), ref1) < 1e-4
        # a different weight pointer triggers a new filter transform
        y = plan.run(xd, w2d, bd)
        torch.cuda.synchronize()
        assert oracle.error_ratio(y.cpu().numpy(), ref2) < 1e-4
        # same pointer, new contents.  The C ABI itself keys the prepared weights on the pointer (raw call: stale) ...
        w2d.data.copy_(wd)                                  # a write the binding's version check does not see
        m.lib.mnn_conv_run(plan._h, xd.data_ptr(), w2d.data_ptr(), bd.data_ptr(), y.data_ptr(), 0)
        torch.cuda.synchronize()
        assert oracle.error_ratio(y.cpu().numpy(), ref2) < 1e-4
        # ... until the caller says so
        plan.invalidate_weights()
        y = plan.run(xd, w2d, bd)
        torch.cuda.synchronize()
        assert oracle.error_ratio(y.cpu().numpy(), ref1) < 1e-4
        # the binding notices an in-place write that torch counts, and prepares the weights again by itself
        w2d.copy_(torch.from_numpy(w2).cuda())
        y = plan.run(xd, w2d, bd)
        torch.cuda.synchronize()
        assert oracle.error_ratio(y.cpu().numpy(), ref2) < 1e-4


def test_inadmissible_forced_schemes_are_refused():
    m = mnn()
    s2 = config_layers(2)[4]
    with pytest.raises(m.MnnError) as e:
        m.ConvPlan.for_layer(s2, options=m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=2, force_variant=0))
    assert e.value.code == -2
    with pytest.raises(m.MnnError) as e:
        m.ConvPlan.for_layer(config_layers(1)[0], options=m.Options(force_kind=m.SCHEME_GEMM1X1))
    assert e.value.code == -2
    with pytest.raises(m.MnnError) as e:     # the fused arrangement multiplies in fp32 only
        m.ConvPlan.for_layer(config_layers(1)[0], options=m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=2,
                                                                     force_prec=m.GEMM_BF16X3, force_variant=1))
    assert e.value.code == -2


def test_run_on_a_side_stream_and_timed_run():
    m = mnn()
    layer = config_layers(2)[1]
    x, w, b = draw(layer)
    xd, wd, bd = (torch.from_numpy(a).cuda() for a in (x, w, b))
    ref = oracle.conv2d(x, w, b, pad=1)
    side = torch.cuda.Stream()
    with m.ConvPlan.for_layer(layer, options=m.Options(force_kind=m.SCHEME_WINOGRAD, force_tile_n=4, force_variant=0)) as plan:
        y = torch.empty(plan.out_shape, device="cuda")
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            plan.run(xd, wd, bd, y, stream=side)
        side.synchronize()
        assert oracle.error_ratio(y.cpu().numpy(), ref) < 1e-4
        ms = plan.run_timed(xd, wd, bd, y, iters=3)
        assert len(ms) == m.STAGE_COUNT and all(v > 0 for v in ms)
        assert oracle.error_ratio(y.cpu().numpy(), ref) < 1e-4


def test_measured_device_peaks():
    """The two probes behind the measured roofline ceilings: the matrix-core issue rate cannot exceed the published
    fp32 figure (256 CUs x 256 FLOP/clk x 2.4 GHz) and a copy kernel cannot exceed the published HBM rate; both must
    be above what the library's own kernels reach."""
    m = mnn()
    p = m.measure_device_peaks()
    assert 1.0e14 < p["mfma_f32_flops"] <= 1.02 * 157.3e12, p
    assert 3.0e12 < p["copy_bytes_per_s"] <= 8.0e12, p


def test_calibration_and_pruned_search():
    """The device model of the analytic cost: calibrated constants are in the range of this chip, and a search
    pruned by the prediction still lands on a scheme about as fast as the exhaustive search's."""
    m = mnn()
    saved = m.get_device_model()
    try:
        model = m.calibrate()
        assert 6e13 < model["flops"] < 1.6e14            # fp32 matrix-core GEMM: 60 .. 157 TFLOP/s
        assert 2e12 < model["bytes_per_s"] < 8e12
        assert 5e-4 < model["t_schedule_ms"] < 3e-2
        assert m.get_device_model() == model
        for layer in (config_layers(3)[1], config_layers(5)[1].with_batch(4)):
            m.cache_clear()
            with m.ConvPlan.for_layer(layer) as full:
                timed_full = [c for c in full.candidates if c.est_ms >= 0]
                best = min(c.est_ms for c in timed_full)
            m.cache_clear()
            with m.ConvPlan.for_layer(layer, options=m.Options(prune_ratio=2.0)) as pruned:
                cands = pruned.candidates
                timed = [c for c in cands if c.est_ms >= 0]
                chosen = pruned.scheme
                mine = [c for c in timed if (c.kind, c.tile_n, c.variant) == (chosen.kind, chosen.tile_n, chosen.variant)]
            assert len(cands) == len(timed_full) and 1 <= len(timed) < len(cands), (len(timed), len(cands))
            assert mine and mine[0].est_ms <= 1.3 * best
            print(f"[prune] {layer.name}: timed {len(timed)} of {len(cands)}, {mine[0].est_ms:.4f} ms vs best {best:.4f} ms", flush=True)
    finally:
        m.set_device_model(**saved)
        m.cache_clear()


def test_saved_pre_inference_results_plan_without_timing(tmp_path):
    """mnn_conv_cache_save / _load: scheme choice (S), GEMM tile configuration (G) and the input transform's wavefront
    cap (I) of a layer survive in a text file; planning the same layer from that file gives the same plan description
    and is much faster than the timed search, and the planned layer still matches the oracle."""
    import time
    m = mnn()
    layer = config_layers(3)[0]                              # 64 channels, 56 x 56, N = 32: a grid long enough for the cap to be tuned
    m.cache_clear()
    t0 = time.perf_counter()
    with m.ConvPlan.for_layer(layer) as plan:
        first, scheme = plan.describe(), plan.scheme
    t_search = time.perf_counter() - t0
    path = tmp_path / "plans.txt"
    m.cache_save(str(path))
    text = path.read_text()
    tags = {line.split()[0] for line in text.splitlines()[1:] if line.strip()}
    assert {"S", "G"} <= tags and (scheme.kind != m.SCHEME_WINOGRAD or "I" in tags)
    m.cache_clear()
    m.cache_load(str(path))
    t0 = time.perf_counter()
    with m.ConvPlan.for_layer(layer) as plan:
        assert plan.describe() == first
        t_cached = time.perf_counter() - t0
        x, w, b = draw(layer)
        y = plan.run(*(torch.from_numpy(a).cuda() for a in (x, w, b)))
        torch.cuda.synchronize()
    assert t_cached < 0.5 * t_search, (t_cached, t_search)
    ref = oracle.conv2d(x, w, b, stride=layer.stride, pad=layer.pad, dil=layer.dil)
    tol = 1e-3 if (scheme.kind == m.SCHEME_WINOGRAD and scheme.tile_n + layer.k_long - 1 > 6) else 1e-4
    assert oracle.error_ratio(y.cpu().numpy(), ref) <= tol
    m.cache_clear()
