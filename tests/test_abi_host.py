"""Host-side checks of the C ABI (no GPU needed): exports, generator, analytic cost, candidate
enumeration, the selection rule and argument validation."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import cook_toom, cost_model

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def mnn():
    import paper_2002_12418_amd as m
    m.lib  # forces the load; raises if the shared object is missing and cannot be built
    return m


def test_every_declared_symbol_is_exported(mnn):
    header = open(os.path.join(ROOT, "include", "mnn_conv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = sorted(set(re.findall(r"\b(mnn_[a-z0-9_]+)\s*\(", header)))
    assert len(names) >= 20
    lib = ctypes.CDLL(mnn.library_path())
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in mnn_conv.h but not exported"


def test_version_and_defaults(mnn):
    assert mnn.version() >= 100
    o = mnn.Options.defaults()
    assert (o.force_kind, o.alpha_max, o.plan_iters, o.use_cache, o.force_variant) == (mnn.SCHEME_AUTO, 10, 10, 1, -1)
    assert o.point_scale_f == 0.0


NK = [(n, k) for k in range(2, 8) for n in range(2, 9) if n + k - 1 <= 12]


@pytest.mark.parametrize("n,k", NK)
@pytest.mark.parametrize("f", [0.5, 1.0, 0.25])
def test_generator_equals_exact_rationals_rounded_once(mnn, n, k, f):
    """The library's host generator (integer symmetric polynomials times powers of f) against the oracle's
    independent exact-rational construction: identical float32 matrices."""
    from fractions import Fraction
    AT, G, BT = mnn.get_transforms(n, k, f)
    AT_q, G_q, BT_q = cook_toom.matrices(n, k, Fraction(f))
    for got, want in ((AT, AT_q), (G, G_q), (BT, BT_q)):
        want32 = cook_toom.to_float(want).astype(np.float32)
        assert got.shape == want32.shape
        np.testing.assert_array_equal(got, want32)


@pytest.mark.parametrize("n,k", [(n, k) for k in range(2, 8) for n in range(2, 9) if n + k - 1 <= 10 and (n + k) % 2 == 1])
@pytest.mark.parametrize("f", [0.5, 0.425, 1.0])
def test_even_alpha_matrices_have_the_sum_and_difference_structure(mnn, n, k, f):
    """What the transform kernels exploit for an even number of points 0, +f, -f, ..., infinity (half the
    multiply-adds): in B^T the row of point 0 is an even polynomial, the row of infinity an odd one, and the rows of +p
    and -p share their even coefficients and have opposite odd ones; in A^T the column of point 0 feeds the first
    output only, the column of infinity the last only, and the columns of +p and -p are equal in even rows and
    opposite in odd ones.  The kernels check this at launch and fall back to the dense product; here it is pinned
    for every generated pair of matrices, so that the fast path is the one the parity tests run."""
    AT, G, BT = mnn.get_transforms(n, k, f)
    a = n + k - 1
    assert a % 2 == 0
    assert np.all(BT[0, 1::2] == 0) and np.all(BT[a - 1, 0::2] == 0)
    for m in range(1, a - 1, 2):
        assert BT[m, 0] == BT[m, a - 1] == BT[m + 1, 0] == BT[m + 1, a - 1] == 0
        sign = np.where(np.arange(1, a - 1) % 2 == 1, -1.0, 1.0).astype(np.float32)
        np.testing.assert_array_equal(BT[m + 1, 1:a - 1], sign * BT[m, 1:a - 1])
    assert np.all(AT[1:, 0] == 0) and np.all(AT[:n - 1, a - 1] == 0)
    rows = np.where(np.arange(n) % 2 == 1, -1.0, 1.0).astype(np.float32)
    for m in range(1, a - 1, 2):
        np.testing.assert_array_equal(AT[:, m + 1], rows * AT[:, m])


def test_generator_rejects_bad_arguments(mnn):
    with pytest.raises(mnn.MnnError) as e:
        mnn.get_transforms(8, 7, 0.5)           # alpha = 14 > 12
    assert e.value.code == -2
    with pytest.raises(mnn.MnnError) as e:
        mnn.get_transforms(2, 3, -1.0)
    assert e.value.code == -1


@pytest.mark.parametrize("shape", [(3, 64, 64, 56, 56), (3, 512, 512, 7, 7), (5, 128, 128, 64, 64), (7, 64, 64, 112, 112),
                                   (2, 3, 16, 223, 223), (3, 16, 16, 32, 32)])
def test_analytic_cost_matches_oracle_model(mnn, shape):
    k, ic, oc, oh, ow = shape
    for n in range(1, 9 - k + 1):
        assert mnn.analytic_cost(k, ic, oc, oh, ow, n) == float(cost_model.plane_cost(n, k, ic, oc, oh, ow))
    for amax in (8, 6, 10):
        if amax >= k:
            assert mnn.analytic_tile(k, ic, oc, oh, ow, amax) == cost_model.best_tile(k, ic, oc, oh, ow, amax)


def test_enumeration_rules(mnn):
    # k = 1, stride 1, no padding -> one matrix multiplication
    c = mnn.enumerate_schemes(16, 32, 112, 112, 64, 1, 1)
    assert all(s.kind == mnn.SCHEME_GEMM1X1 for s in c)
    assert [s.variant for s in c] == [0, 1]               # plain and one level of Strassen (the rule stops at 32 x 16)
    c = mnn.enumerate_schemes(16, 256, 14, 14, 512, 1, 1)
    assert [(s.kind, s.variant) for s in c] == [(mnn.SCHEME_GEMM1X1, v) for v in (0, 1, 2)]
    c = mnn.enumerate_schemes(3, 19, 7, 7, 21, 1, 1)       # nothing divides: the plain product only
    assert [(s.kind, s.variant) for s in c] == [(mnn.SCHEME_GEMM1X1, 0)]
    # stride 2 / dilation 2 -> sliding window only
    for kw in (dict(stride=2, pad=1), dict(dil=2, pad=2)):
        c = mnn.enumerate_schemes(1, 64, 56, 56, 128, 3, 3, **kw)
        assert [s.kind for s in c] == [mnn.SCHEME_DIRECT]
    # k_h x k_w with several taps on both axes: sliding window + F(n, .) with n x n tiles while the larger alpha is <= 8
    c = mnn.enumerate_schemes(1, 8, 20, 20, 8, 3, 5)
    assert c[0].kind == mnn.SCHEME_DIRECT
    assert [(s.kind, s.tile_n, s.variant) for s in c[1:]] == [(mnn.SCHEME_WINOGRAD, n, mnn.WINO_UNFUSED) for n in (2, 3, 4)]
    c = mnn.enumerate_schemes(1, 8, 20, 20, 8, 3, 5, options=mnn.Options(alpha_max=8))       # the default already stops at alpha = 8 for these
    assert [s.tile_n for s in c[1:]] == [2, 3, 4]
    c = mnn.enumerate_schemes(1, 8, 20, 20, 8, 2, 9)                                           # more than 7 taps on an axis
    assert [s.kind for s in c] == [mnn.SCHEME_DIRECT]
    c = mnn.enumerate_schemes(1, 8, 20, 20, 8, 1, 7, stride=(1, 2))
    assert [s.kind for s in c] == [mnn.SCHEME_DIRECT]
    # a single row or column of k taps: sliding window + one-dimensional F(n, k), unfused only
    for kh, kwid in ((1, 7), (7, 1)):
        c = mnn.enumerate_schemes(1, 8, 20, 20, 8, kh, kwid)
        assert c[0].kind == mnn.SCHEME_DIRECT
        assert [(s.kind, s.tile_n, s.variant) for s in c[1:]] == [(mnn.SCHEME_WINOGRAD, n, mnn.WINO_UNFUSED) for n in (2, 3, 4)]
        c = mnn.enumerate_schemes(1, 8, 20, 20, 8, kh, kwid, options=mnn.Options(alpha_max=8))
        assert [(s.kind, s.tile_n, s.variant) for s in c[1:]] == [(mnn.SCHEME_WINOGRAD, 2, mnn.WINO_UNFUSED)]
    c = mnn.enumerate_schemes(1, 8, 20, 20, 8, 3, 1, pad=(1, 0))
    assert [(s.tile_n, s.variant) for s in c if s.kind == mnn.SCHEME_WINOGRAD] == [(n, mnn.WINO_UNFUSED) for n in range(2, 9)]
    # 3x3 stride 1: sliding window + F(n,3) for n = 2..8 (alpha <= 10), each in its kernel arrangements
    c = mnn.enumerate_schemes(1, 64, 56, 56, 64, 3, 3, pad=1)
    assert c[0].kind == mnn.SCHEME_DIRECT
    wino = [s for s in c if s.kind == mnn.SCHEME_WINOGRAD]
    assert sorted({s.tile_n for s in wino}) == [2, 3, 4, 5, 6, 7, 8]
    assert all(any(s.tile_n == n and s.variant == mnn.WINO_UNFUSED for s in wino) for n in range(2, 9))
    assert all(s.est_ms < 0 for s in c)
    # alpha_max caps n; 7x7 with alpha <= 8 only admits n = 2
    c = mnn.enumerate_schemes(1, 64, 56, 56, 64, 3, 3, pad=1, options=mnn.Options(alpha_max=6))
    assert sorted({s.tile_n for s in c if s.kind == mnn.SCHEME_WINOGRAD}) == [2, 3, 4]
    c = mnn.enumerate_schemes(16, 64, 112, 112, 64, 7, 7, pad=3, options=mnn.Options(alpha_max=8))
    assert sorted({s.tile_n for s in c if s.kind == mnn.SCHEME_WINOGRAD}) == [2]
    c = mnn.enumerate_schemes(16, 64, 112, 112, 64, 7, 7, pad=3)
    assert sorted({s.tile_n for s in c if s.kind == mnn.SCHEME_WINOGRAD}) == [2, 3, 4]
    # 1x1 with padding is not the plain GEMM case
    c = mnn.enumerate_schemes(1, 8, 8, 8, 8, 1, 1, pad=1)
    assert [s.kind for s in c] == [mnn.SCHEME_DIRECT]


def test_selection_rule(mnn):
    S = mnn.Scheme
    W, D = mnn.SCHEME_WINOGRAD, mnn.SCHEME_DIRECT
    # plain argmin
    c = [S(D, 0, 0, 0, 1.0), S(W, 2, 0, 0, 0.5), S(W, 4, 0, 0, 0.3), S(W, 6, 0, 0, 0.4)]
    assert mnn.select_scheme(c, 3) == 2
    # within 2 % of the best: the smaller alpha wins
    c = [S(D, 0, 0, 0, 1.0), S(W, 2, 0, 0, 0.303), S(W, 4, 0, 0, 0.300), S(W, 6, 0, 0, 0.301)]
    assert mnn.select_scheme(c, 3) == 1
    # ... but not beyond 2 %
    c = [S(W, 2, 0, 0, 0.310), S(W, 4, 0, 0, 0.300)]
    assert mnn.select_scheme(c, 3) == 1
    # untimed candidates are ignored; sliding window counts as alpha = k
    c = [S(D, 0, 0, 0, 0.2), S(W, 2, 0, 0, -1.0), S(W, 4, 0, 0, 0.2)]
    assert mnn.select_scheme(c, 3) == 0
    # same alpha: fp32 before bf16, then the faster arrangement
    c = [S(W, 4, 1, 0, 0.100), S(W, 4, 0, 1, 0.1005), S(W, 4, 0, 0, 0.101)]
    assert mnn.select_scheme(c, 3) == 1
    with pytest.raises(mnn.MnnError):
        mnn.select_scheme([S(W, 2, 0, 0, -1.0)], 3)


def test_selection_is_deterministic(mnn):
    rng = np.random.default_rng(0)
    for _ in range(50):
        c = [mnn.Scheme(mnn.SCHEME_WINOGRAD, int(n), 0, int(v), float(t))
             for n, v, t in zip(rng.integers(2, 7, 8), rng.integers(0, 3, 8), rng.uniform(0.1, 0.2, 8))]
        first = mnn.select_scheme(c, 3)
        assert all(mnn.select_scheme(c, 3) == first for _ in range(3))
        best = min(s.est_ms for s in c)
        assert c[first].est_ms <= best * 1.02 * (1 + 1e-6)


def test_plan_argument_validation(mnn):
    import torch
    bad = [
        dict(n=0, c_in=1, h=4, w=4, c_out=1, kh=3, kw=3),            # empty batch
        dict(n=1, c_in=1, h=2, w=2, c_out=1, kh=3, kw=3),            # kernel larger than the image
        dict(n=1, c_in=1, h=4, w=4, c_out=1, kh=3, kw=3, stride=0),
        dict(n=1, c_in=1, h=4, w=4, c_out=1, kh=3, kw=3, pad=-1),
    ]
    for kw in bad:
        with pytest.raises(mnn.MnnError) as e:
            mnn.ConvPlan(**kw)
        assert e.value.code == -1, kw
    with pytest.raises(mnn.MnnError) as e:
        mnn.enumerate_schemes(1, 8, 8, 8, 8, 3, 3, options=mnn.Options(alpha_max=11))
    assert e.value.code == -2
    if not torch.cuda.is_available():
        with pytest.raises(mnn.MnnError) as e:
            mnn.ConvPlan(1, 4, 8, 8, 4, 3, 3, pad=1)
        assert e.value.code == -5                                     # MNN_E_NO_DEVICE, never a CPU fallback
        assert "device" in str(e.value).lower()
        with pytest.raises(mnn.MnnError) as e:
            mnn.measure_device_peaks()
        assert e.value.code == -5
    assert mnn.lib.mnn_measure_device_peaks(None, None) == -1          # NULL out


def test_gemm_variant_table(mnn):
    for prec in (mnn.GEMM_FP32, mnn.GEMM_BF16, mnn.GEMM_BF16X3):
        names = mnn.gemm_variants(prec)
        assert names[0] == "auto" and len(names) == len(set(names)) and len(names) > 4
    assert mnn.gemm_variants(7) == []


def test_enumeration_with_bf16_allowed(mnn):
    c = mnn.enumerate_schemes(1, 64, 56, 56, 64, 3, 3, pad=1, options=mnn.Options(allow_bf16=1))
    x3 = [s for s in c if s.prec == mnn.GEMM_BF16X3]
    plain = [s for s in c if s.prec == mnn.GEMM_BF16]
    # split-operand variant for the sliding window and every F(n,3); plain bf16 only for the sliding window
    assert sorted(s.tile_n for s in x3) == [0, 2, 3, 4, 5, 6, 7, 8] and all(s.variant == 0 for s in x3)
    assert [(s.kind, s.tile_n) for s in plain] == [(mnn.SCHEME_DIRECT, 0)]
    c = mnn.enumerate_schemes(16, 32, 112, 112, 64, 1, 1, options=mnn.Options(allow_bf16=1))
    assert [(s.kind, s.prec, s.variant) for s in c] == [(mnn.SCHEME_GEMM1X1, 0, 0), (mnn.SCHEME_GEMM1X1, 2, 0),
                                                        (mnn.SCHEME_GEMM1X1, 1, 0), (mnn.SCHEME_GEMM1X1, 0, 1)]


def test_product_path_does_not_import_the_oracle():
    """The package, bench hot path and C sources must not reference the oracle."""
    pkg = os.path.join(ROOT, "paper_2002_12418_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "oracle/" not in text, f
    for dirpath, _, files in os.walk(os.path.join(ROOT, "oracle")):
        for f in files:
            if f.endswith((".py", ".c")):
                text = open(os.path.join(dirpath, f)).read()
                assert "paper_2002_12418_amd" not in text and "mnn_conv" not in text, f


def test_cache_file_round_trip_rejects_garbage(mnn, tmp_path):
    good = tmp_path / "plans.txt"
    mnn.cache_clear()
    mnn.cache_save(str(good))
    assert good.read_text().startswith("mnnconv-plan-cache 3")
    mnn.cache_load(str(good))
    assert mnn.cache_size() == 0
    # a hand-written entry: device 0, cfg1 layer with the default options, F(4,3) unfused
    good.write_text("mnnconv-plan-cache 3\nS 0 16 1 16 32 32 16 3 3 1 1 1 1 1 1 8 0 0 0.5 | 2 4 0 0 0.01\n")
    mnn.cache_load(str(good))
    assert mnn.cache_size() == 1
    mnn.cache_clear()
    bad = tmp_path / "bad.txt"
    bad.write_text("something else\n")
    with pytest.raises(mnn.MnnError):
        mnn.cache_load(str(bad))
    with pytest.raises(mnn.MnnError):
        mnn.cache_load(str(tmp_path / "missing.txt"))


def test_strassen_rule_matches_oracle(mnn):
    """Levels the library allows = the paper's inequality (oracle.cost_model) at every level, cut where the
    halves would lose 16-byte rows (M, ncols divisible by 8, R by 2 before each halving)."""
    def expected(M, R, N, cap):
        lv = 0
        while lv < cap and M % 8 == 0 and N % 8 == 0 and R % 2 == 0 and cost_model.strassen_should_recurse(M, R, N):
            M, R, N, lv = M // 2, R // 2, N // 2, lv + 1
        return lv
    for shape in [(1024, 1024, 784), (1024, 512, 784), (256, 256, 256), (512, 512, 1024), (64, 32, 200704),
                  (24, 6, 24), (8, 2, 8), (16, 16, 16), (32, 32, 32), (30, 30, 30), (40, 12, 56), (1024, 1024, 788)]:
        for cap in (0, 1, 2, 4):
            assert mnn.strassen_levels_by_rule(shape[0], shape[1], shape[2], cap) == expected(*shape, cap), (shape, cap)
    # the paper's Table 3 sizes all pass the rule at the first level
    for n in (256, 512, 1024):
        assert mnn.strassen_levels_by_rule(n, n, n, 1) == 1


def test_device_cost_model(mnn):
    """Section 3.2 (2): per kernel work / FLOPS + t_schedule, with the memory side added.  Checked against the
    formula written out here for an unfused F(4,3) layer and a sliding-window layer, under a model with round
    numbers; then the default model's constants are restored."""
    saved = mnn.get_device_model()
    try:
        mnn.set_device_model(1e14, 4e12, 0.01)
        N, C, H, K, k, n = 32, 128, 28, 128, 3, 4
        a, P = n + k - 1, N * 7 * 7
        x_b, y_b = 4.0 * N * C * H * H, 4.0 * N * K * H * H
        kernels = [(2.0 * 2 * a ** 3 * C * P, x_b + 4.0 * a * a * C * P),
                   (2.0 * a * a * K * C * P, 4.0 * a * a * (K * C + C * P + K * P)),
                   (2.0 * (n * a * a + n * n * a) * K * P, 4.0 * a * a * K * P + y_b)]
        want = sum(max(f / 1e14, b / 4e12) * 1e3 + 0.01 for f, b in kernels)
        got = mnn.predict_ms(N, C, H, H, K, k, k, mnn.Scheme(mnn.SCHEME_WINOGRAD, n, mnn.GEMM_FP32, mnn.WINO_UNFUSED, -1.0), pad=1)
        assert got == pytest.approx(want, rel=1e-12)
        direct = mnn.predict_ms(N, C, H, H, K, k, k, mnn.Scheme(mnn.SCHEME_DIRECT, 0, mnn.GEMM_FP32, 0, -1.0), pad=1)
        assert direct == pytest.approx(max(2.0 * N * K * C * H * H * 9 / 1e14, (x_b + y_b + 4.0 * K * C * 9) / 4e12) * 1e3 + 0.01, rel=1e-12)
        # a launch-bound layer: three kernels cost three schedule terms, one kernel one
        tiny_w = mnn.predict_ms(1, 16, 8, 8, 16, 3, 3, mnn.Scheme(mnn.SCHEME_WINOGRAD, 2, 0, 0, -1.0), pad=1)
        tiny_d = mnn.predict_ms(1, 16, 8, 8, 16, 3, 3, mnn.Scheme(mnn.SCHEME_DIRECT, 0, 0, 0, -1.0), pad=1)
        assert tiny_w > 0.03 and 0.01 < tiny_d < 0.011
        with pytest.raises(mnn.MnnError):
            mnn.set_device_model(0.0, 1.0, 0.0)
        with pytest.raises(mnn.MnnError):
            mnn.predict_ms(1, 16, 8, 8, 16, 3, 3, mnn.Scheme(mnn.SCHEME_GEMM1X1, 0, 0, 0, -1.0))
    finally:
        mnn.set_device_model(**saved)
    assert mnn.get_device_model() == saved
    with pytest.raises(mnn.MnnError):
        mnn.enumerate_schemes(1, 16, 8, 8, 16, 3, 3, options=mnn.Options(prune_ratio=0.5))
