"""Chained execution (preparation-execution decoupling, Section 3.2 / Table 2): a chain of layers planned once,
one arena with lifetime-based reuse, eager run and HIP-graph replay.

Checks: the chain's result against the float64 oracle applied layer after layer (activations rounded to
float32 between layers, as the device stores them); bit-identity with the same layers run one by one through
mnn_conv_run (same kernels, so sharing memory must change nothing); every graph replay against the eager
result, with eager work and synchronisation between replays; the arena's bookkeeping.

Tolerance of the end-to-end comparison: each layer is within 1e-4 (fp32 schemes with alpha <= 6; 1e-3 above)
of the definition, and a relative perturbation of a layer's input passes to its output at most at about the
same relative size (He-normal weights keep the scale), so L layers stay within L times the per-layer bound.
"""
import numpy as np
import pytest
import torch

import oracle
from conv_workloads import chain_layers, draw

pytestmark = pytest.mark.gpu


def mnn():
    import paper_2002_12418_amd as m
    return m


def draw_chain(layers):
    x0 = draw(layers[0])[0]
    wb = [draw(l)[1:] for l in layers]
    return x0, wb


def oracle_chain(layers, x0, wb):
    acts = []
    x = x0
    for l, (w, b) in zip(layers, wb):
        y = oracle.conv2d(x, w, b, stride=l.stride, pad=l.pad, dil=l.dil)
        acts.append(y)
        x = y.astype(np.float32)
    return acts


def load_chain(m, layers, wb, options=None):
    ch = m.ConvChain(layers, options=options)
    keep = []
    for i, (w, b) in enumerate(wb):
        wd, bd = torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda()
        ch.set_weights(i, wd, bd)
        keep.append((wd, bd))
    torch.cuda.synchronize()
    return ch, keep


def bound(m, ch, n_layers):
    per_layer = 0.0
    for i in range(n_layers):
        s = ch.scheme(i)
        alpha = s.tile_n + ch.layers[i].kh - 1 if s.kind == m.SCHEME_WINOGRAD else 0
        per_layer += 1e-3 if alpha > 6 else 1e-4
    return per_layer


@pytest.mark.parametrize("kind,n", [("small", 2), ("resnet18_trunk", 1), ("resnet18_trunk", 3)])
def test_chain_matches_oracle_and_layerwise_runs(kind, n):
    m = mnn()
    layers = chain_layers(kind, n)
    x0, wb = draw_chain(layers)
    ref = oracle_chain(layers, x0, wb)
    ch, keep = load_chain(m, layers, wb)
    xd = torch.from_numpy(x0).cuda()
    y = ch.run(xd)
    torch.cuda.synchronize()
    err = oracle.error_ratio(y.cpu().numpy(), ref[-1])
    assert err <= bound(m, ch, len(layers)), (kind, n, err, [ch.describe(i) for i in range(len(layers))])
    # the last intermediate activation is still in the arena (nothing alive with it has been placed over it)
    a = ch.activation_to_numpy(len(layers) - 2)
    assert oracle.error_ratio(a, ref[-2]) <= bound(m, ch, len(layers) - 1)

    # the same layers one at a time, each plan with memory of its own: identical bits
    cur = xd
    for i, l in enumerate(layers):
        with m.ConvPlan.for_layer(l) as plan:
            s_chain, s_plan = ch.scheme(i), plan.scheme
            assert (s_chain.kind, s_chain.tile_n, s_chain.prec, s_chain.variant) == \
                   (s_plan.kind, s_plan.tile_n, s_plan.prec, s_plan.variant)
            assert ch.describe(i) == plan.describe()
            cur = plan.run(cur, keep[i][0], keep[i][1])
            torch.cuda.synchronize()
    assert torch.equal(cur, y)

    info = ch.info
    assert info["n_layers"] == len(layers)
    assert info["live_peak_bytes"] <= info["arena_bytes"] < info["unshared_bytes"]
    ch.close()


def test_graph_replays_equal_eager_runs():
    m = mnn()
    layers = chain_layers("resnet18_trunk", 1)
    x0, wb = draw_chain(layers)
    ch, keep = load_chain(m, layers, wb)
    xd = torch.from_numpy(x0).cuda()
    y_eager = ch.run(xd).clone()
    torch.cuda.synchronize()

    xg = xd.clone()
    yg = ch.capture(xg)
    info = ch.info
    assert info["graph_nodes"] == info["kernels_per_run"] > 0
    rng = np.random.default_rng(7)
    for rep in range(4):
        if rep:
            # new contents at the captured address; eager reference for them, more eager work, a sync
            xn = torch.from_numpy(rng.uniform(-1, 1, x0.shape).astype(np.float32)).cuda()
            y_eager = ch.run(xn).clone()
            xg.copy_(xn)
            _ = (xn * 2).sum().item()
        yg.fill_(float("nan"))
        ch.replay()
        torch.cuda.synchronize()
        assert torch.equal(yg, y_eager), f"replay {rep}"
    # two replays back to back without host synchronisation in between
    ch.replay()
    ch.replay()
    torch.cuda.synchronize()
    assert torch.equal(yg, y_eager)
    ch.close()


def test_forced_direct_chain_and_no_bias():
    m = mnn()
    layers = chain_layers("small", 1)
    x0, wb = draw_chain(layers)
    wb = [(w, None) if i % 2 else (w, b) for i, (w, b) in enumerate(wb)]
    ref = oracle_chain(layers, x0, wb)
    o = m.Options.defaults()
    o.force_kind = m.SCHEME_DIRECT
    ch = m.ConvChain(layers, options=o)
    keep = []
    for i, (w, b) in enumerate(wb):
        wd = torch.from_numpy(w).cuda()
        bd = None if b is None else torch.from_numpy(b).cuda()
        ch.set_weights(i, wd, bd)
        keep.append((wd, bd))
    assert all(ch.scheme(i).kind == m.SCHEME_DIRECT for i in range(len(layers)))
    y = ch.run(torch.from_numpy(x0).cuda())
    torch.cuda.synchronize()
    assert oracle.error_ratio(y.cpu().numpy(), ref[-1]) <= 1e-4 * len(layers)
    ch.close()


def test_chain_call_order_errors():
    m = mnn()
    layers = chain_layers("small", 1)
    x0, wb = draw_chain(layers)
    ch = m.ConvChain(layers)
    xd = torch.from_numpy(x0).cuda()
    with pytest.raises(m.MnnError) as e:
        ch.run(xd)
    assert "weights of layer 0" in str(e.value)
    with pytest.raises(m.MnnError):
        ch.replay()
    with pytest.raises(m.MnnError):
        ch.capture(xd)
    with pytest.raises(ValueError):
        ch.set_weights(0, torch.zeros(3, 3, device="cuda"))
    ch.close()


def test_chain_on_a_side_stream_and_with_bf16_operands():
    """The chain enqueues on the stream it is given (eager and graph replay), and carries the planner's options:
    with allow_bf16 the layers may take split-bf16 operands and the result stays within the bf16 bound."""
    m = mnn()
    layers = chain_layers("resnet18_trunk", 2)
    x0, wb = draw_chain(layers)
    ref = oracle_chain(layers, x0, wb)
    side = torch.cuda.Stream()
    for options, tol in ((None, None), (m.Options(allow_bf16=1), 2e-2)):
        m.cache_clear()
        ch = m.ConvChain(layers, options=options, stream=side)
        keep = []
        for i, (w, b) in enumerate(wb):
            wd, bd = torch.from_numpy(w).cuda(), torch.from_numpy(b).cuda()
            keep.append((wd, bd))
        torch.cuda.synchronize()
        for i, (wd, bd) in enumerate(keep):
            ch.set_weights(i, wd, bd, stream=side)
        xd = torch.from_numpy(x0).cuda()
        torch.cuda.synchronize()
        y = torch.empty(layers[-1].out_shape, device="cuda")
        ch.run(xd, y, stream=side)
        side.synchronize()
        y_eager = y.clone()
        err = oracle.error_ratio(y_eager.cpu().numpy(), ref[-1])
        assert err <= (tol if tol is not None else bound(m, ch, len(layers))), err
        yg = ch.capture(xd)
        ch.replay(stream=side)
        side.synchronize()
        assert torch.equal(yg, y_eager)
        ch.close()
    m.cache_clear()
