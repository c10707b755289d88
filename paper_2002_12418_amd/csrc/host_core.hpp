// Errors, layer validation, options, candidate enumeration, the analytic cost of Section 3.2 (1)
// and the selection rule.
// Private part of api.cpp (included there once, in order); everything lives in its unnamed namespace.
#pragma once

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

int fail_hip(hipError_t e, const char* what)
{
    // hipGetLastError clears the sticky error so that one failure is not reported twice
    (void)hipGetLastError();
    if (e == hipErrorOutOfMemory) return fail(MNN_E_OOM, "%s: %s", what, hipGetErrorString(e));
    return fail(MNN_E_HIP, "%s: %s", what, hipGetErrorString(e));
}

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

void default_options(mnn_conv_options* o)
{
    o->force_kind = MNN_SCHEME_AUTO;
    o->force_tile_n = 0;
    o->force_prec = MNN_GEMM_FP32;
    o->force_variant = -1;
    o->allow_bf16 = 0;
    o->alpha_max = kMaxAlphaT;
    o->point_scale_f = 0.f;
    o->plan_warmup = 2;
    o->plan_iters = 10;
    o->use_cache = 1;
    o->prune_ratio = 0.f;
}

struct Layer {
    mnn_conv_shape s;
    mnn_conv_geom g;
    int Ho, Wo;
};

int validate(const mnn_conv_shape* shape, const mnn_conv_geom* geom, Layer* L)
{
    if (!shape || !geom) return fail(MNN_E_INVALID_ARG, "shape and geom must not be NULL");
    const mnn_conv_shape& s = *shape;
    const mnn_conv_geom& g = *geom;
    if (s.n <= 0 || s.c_in <= 0 || s.h <= 0 || s.w <= 0 || s.c_out <= 0 || s.kh <= 0 || s.kw <= 0)
        return fail(MNN_E_INVALID_ARG, "all shape entries must be positive");
    if (g.stride_h <= 0 || g.stride_w <= 0 || g.dil_h <= 0 || g.dil_w <= 0 || g.pad_h < 0 || g.pad_w < 0)
        return fail(MNN_E_INVALID_ARG, "stride and dilation must be positive, padding non-negative");
    const long long eh = (long long)s.h + 2ll * g.pad_h - (long long)g.dil_h * (s.kh - 1) - 1;
    const long long ew = (long long)s.w + 2ll * g.pad_w - (long long)g.dil_w * (s.kw - 1) - 1;
    if (eh < 0 || ew < 0) return fail(MNN_E_INVALID_ARG, "kernel extent exceeds the padded input: empty output");
    L->s = s;
    L->g = g;
    L->Ho = (int)(eh / g.stride_h) + 1;
    L->Wo = (int)(ew / g.stride_w) + 1;
    const long long in_elems = (long long)s.n * s.c_in * s.h * s.w;
    const long long out_elems = (long long)s.n * s.c_out * L->Ho * L->Wo;
    const long long w_elems = (long long)s.c_out * s.c_in * s.kh * s.kw;
    if (in_elems >= (1ll << 40) || out_elems >= (1ll << 40) || w_elems >= (1ll << 31))
        return fail(MNN_E_UNSUPPORTED, "tensor too large");
    return MNN_OK;
}

int validate_options(const mnn_conv_options* in, mnn_conv_options* o)
{
    if (in) *o = *in; else default_options(o);
    if (o->alpha_max <= 0) o->alpha_max = kMaxAlphaT;
    if (o->alpha_max > kMaxAlphaT)
        return fail(MNN_E_UNSUPPORTED, "alpha_max above %d: the fp32 error of larger tiles exceeds 1e-3", kMaxAlphaT);
    if (!(o->point_scale_f >= 0.f)) return fail(MNN_E_INVALID_ARG, "point_scale_f must be positive (or 0: chosen per alpha)");
    if (o->plan_warmup < 0 || o->plan_iters <= 0) return fail(MNN_E_INVALID_ARG, "plan_warmup >= 0 and plan_iters > 0 required");
    if (o->force_kind < MNN_SCHEME_AUTO || o->force_kind > MNN_SCHEME_GEMM1X1)
        return fail(MNN_E_INVALID_ARG, "unknown force_kind %d", o->force_kind);
    if (o->force_prec < MNN_GEMM_FP32 || o->force_prec > MNN_GEMM_BF16X3)
        return fail(MNN_E_INVALID_ARG, "unknown force_prec %d", o->force_prec);
    if (o->force_variant < -1 || o->force_variant >= MNN_WINO_VARIANTS)
        return fail(MNN_E_INVALID_ARG, "unknown force_variant %d", o->force_variant);
    if (!(o->prune_ratio == 0.f || o->prune_ratio > 1.f)) return fail(MNN_E_INVALID_ARG, "prune_ratio must be 0 or above 1");
    return MNN_OK;
}

bool is_pointwise(const Layer& L)
{
    return L.s.kh == 1 && L.s.kw == 1 && L.g.stride_h == 1 && L.g.stride_w == 1 && L.g.pad_h == 0 && L.g.pad_w == 0;
}

// kernels that are not square: a single row or column (1 x k, k x 1: one-dimensional Winograd along the long axis)
// or several taps on both axes (k_h x k_w: one generated matrix set per axis, n x n output tiles)
bool winograd_rect(const Layer& L)
{
    return L.s.kh != L.s.kw;
}

// output tile extent along an axis with k taps when the scheme's tile is n
int wino_axis_n(int k, int n) { return k == 1 ? 1 : n; }

bool winograd_admissible(const Layer& L)
{
    const bool shape_ok = (L.s.kh == L.s.kw && L.s.kh >= 2) || winograd_rect(L);
    return shape_ok && L.g.stride_h == 1 && L.g.stride_w == 1 && L.g.dil_h == 1 && L.g.dil_w == 1;
}

// whether the transform kernels of F(n, .) exist for this layer's kernel shape
bool wino_tile_available(const Layer& L, int n)
{
    if (winograd_rect(L))
        return winograd_rect_kernels_available(wino_axis_n(L.s.kh, n), L.s.kh, wino_axis_n(L.s.kw, n), L.s.kw);
    return winograd_kernels_available(n, L.s.kh);
}

int wino_k(const Layer& L) { return L.s.kh > L.s.kw ? L.s.kh : L.s.kw; }    // taps along the transformed axis

mnn_scheme make_scheme(int kind, int n, int prec, int variant = 0)
{
    mnn_scheme s;
    s.kind = kind; s.tile_n = n; s.prec = prec; s.variant = variant; s.est_ms = -1.f;
    return s;
}

bool wino_variant_available(int n, int k, int variant)
{
    if (!winograd_kernels_available(n, k)) return false;
    switch (variant) {
        case MNN_WINO_UNFUSED: return true;
        case MNN_WINO_FUSED_OUT_32: return wino_fused_available(n, k);
        case MNN_WINO_FUSED_OUT_64: return wino_fused_has_big_block(n, k);
        default: return false;
    }
}

void push_wino_variants(std::vector<mnn_scheme>* out, int n, int k, int prec)
{
    for (int v = 0; v < MNN_WINO_VARIANTS; ++v)
        if (wino_variant_available(n, k, v)) out->push_back(make_scheme(MNN_SCHEME_WINOGRAD, n, prec, v));
}

// Recursion rule of Section 3.3.2 for [n,k] x [k,m]: go one level down while the multiplications saved exceed
// the additions added,  mnk - 7 (m/2)(n/2)(k/2) > 4 (m/2)(k/2) + 4 (n/2)(k/2) + 7 (m/2)(n/2)  -- compared
// in eighths to stay in integers -- and, here, while the halves keep the 16-byte granularity of the kernels.
bool strassen_rule(long long n, long long k, long long m)
{
    return 8 * m * n * k - 7 * m * n * k > 8 * (m * k + n * k) + 14 * m * n;
}

int strassen_levels(int M, int R, int N, int max_levels)
{
    int l = 0;
    long long m = M, r = R, n = N;
    while (l < max_levels && m % 8 == 0 && n % 8 == 0 && r % 2 == 0 && strassen_rule(m, r, n)) {
        m /= 2; r /= 2; n /= 2;
        ++l;
    }
    return l;
}

// Section 3.2 (1): k = 1 -> matrix multiplication; k > 1 -> sliding window or F(n,k).
std::vector<mnn_scheme> enumerate(const Layer& L, const mnn_conv_options& o)
{
    std::vector<mnn_scheme> out;
    const int base = is_pointwise(L) ? MNN_SCHEME_GEMM1X1 : MNN_SCHEME_DIRECT;
    out.push_back(make_scheme(base, 0, MNN_GEMM_FP32));
    if (o.allow_bf16) {
        out.push_back(make_scheme(base, 0, MNN_GEMM_BF16X3));
        out.push_back(make_scheme(base, 0, MNN_GEMM_BF16));
    }
    if (is_pointwise(L)) {
        // Section 3.3.2: the large matrix multiplication with 1 or 2 levels of Strassen, where the paper's rule
        // says the recursion pays and the halves keep 16-byte rows; variant = number of levels
        const long long cols = (long long)L.s.n * L.s.h * L.s.w;
        for (int lv = 1; lv <= 2 && cols < (1ll << 31); ++lv)
            if (strassen_levels(L.s.c_out, L.s.c_in, (int)cols, lv) == lv && L.s.c_out % 4 == 0 && (L.s.h * L.s.w) % 4 == 0)
                out.push_back(make_scheme(MNN_SCHEME_GEMM1X1, 0, MNN_GEMM_FP32, lv));
        return out;
    }
    if (winograd_admissible(L)) {
        const int k = wino_k(L);
        for (int n = 2; n + k - 1 <= o.alpha_max; ++n) {
            if (winograd_rect(L)) {          // transforms and GEMM as separate kernels only
                if (wino_tile_available(L, n)) {
                    out.push_back(make_scheme(MNN_SCHEME_WINOGRAD, n, MNN_GEMM_FP32, MNN_WINO_UNFUSED));
                    if (o.allow_bf16) out.push_back(make_scheme(MNN_SCHEME_WINOGRAD, n, MNN_GEMM_BF16X3, MNN_WINO_UNFUSED));
                }
                continue;
            }
            push_wino_variants(&out, n, k, MNN_GEMM_FP32);
            if (o.allow_bf16 && winograd_kernels_available(n, k))
                out.push_back(make_scheme(MNN_SCHEME_WINOGRAD, n, MNN_GEMM_BF16X3, MNN_WINO_UNFUSED));
        }
    }
    return out;
}

double analytic_cost(int k, int ic, int oc, int oh, int ow, int n)
{
    const double a = n + k - 1;
    const double blocks = (double)((oh + n - 1) / n) * (double)((ow + n - 1) / n);
    return blocks * (2.0 * ic * a * a * a + (double)ic * oc * a * a + (double)n * a * (2.0 * n + k - 1));
}

int analytic_tile(int k, int ic, int oc, int oh, int ow, int alpha_max)
{
    int best = 1;
    double bc = analytic_cost(k, ic, oc, oh, ow, 1);
    for (int n = 2; n + k - 1 <= alpha_max; ++n) {
        const double c = analytic_cost(k, ic, oc, oh, ow, n);
        if (c < bc) { bc = c; best = n; }
    }
    return best;
}

}  // namespace
