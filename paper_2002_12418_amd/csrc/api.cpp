// C ABI, plan objects and the pre-inference planner (Section 3.2 of the MNN
// paper: computation scheme selection + preparation-execution decoupling).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <cmath>
#include <map>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <tuple>
#include <vector>

#include "../../include/mnn_conv.h"
#include "cook_toom_gen.hpp"
#include "arena.hpp"
#include "kernels.hpp"

using namespace mnnconv;

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
    o->alpha_max = 8;
    o->point_scale_f = 0.5f;
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
    if (o->alpha_max <= 0) o->alpha_max = 8;
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

// kernels with a single row or column (1 x k, k x 1, k >= 2): one-dimensional Winograd along the long axis
bool winograd_rect(const Layer& L)
{
    return (L.s.kh == 1) != (L.s.kw == 1);
}

bool winograd_admissible(const Layer& L)
{
    const bool shape_ok = (L.s.kh == L.s.kw && L.s.kh >= 2) || winograd_rect(L);
    return shape_ok && L.g.stride_h == 1 && L.g.stride_w == 1 && L.g.dil_h == 1 && L.g.dil_w == 1;
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
                if (winograd_kernels_available(n, k)) {
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

// ------------------------------------------------------------------ device cost model (Section 3.2 (2))
// C_op = work / FLOPS + t_schedule per kernel, with the memory side added.  Defaults: measured on MI355X.
std::mutex g_model_mu;
mnn_device_model g_model = {115e12, 4.4e12, 0.005};

struct KernelWork { double flops, bytes; };

// the kernels one inference of `s` launches for layer L, with their algorithmic work
std::vector<KernelWork> scheme_kernels(const Layer& L, const mnn_scheme& s)
{
    const double N = L.s.n, C = L.s.c_in, K = L.s.c_out, H = L.s.h, W = L.s.w, Ho = L.Ho, Wo = L.Wo;
    const double in_b = 4.0 * N * C * H * W, out_b = 4.0 * N * K * Ho * Wo, w_b = 4.0 * K * C * L.s.kh * L.s.kw;
    std::vector<KernelWork> v;
    if (s.kind == MNN_SCHEME_WINOGRAD) {
        const bool rect = winograd_rect(L);
        const double n = s.tile_n, k = wino_k(L), a = n + k - 1;
        const double nh = (rect && L.s.kh == 1) ? 1 : n, nw = (rect && L.s.kw == 1) ? 1 : n;
        const double ah = (rect && L.s.kh == 1) ? 1 : a, aw = (rect && L.s.kw == 1) ? 1 : a;
        const double P = N * std::ceil(Ho / nh) * std::ceil(Wo / nw), a2 = ah * aw;
        v.push_back(KernelWork{2.0 * (ah * ah * aw + ah * aw * aw) * C * P, in_b + 4.0 * a2 * C * P});
        if (s.variant == MNN_WINO_UNFUSED) {
            v.push_back(KernelWork{2.0 * a2 * K * C * P, 4.0 * a2 * (K * C + C * P + K * P)});
            v.push_back(KernelWork{2.0 * (nh * ah * aw + nh * nw * aw) * K * P, 4.0 * a2 * K * P + out_b});
        } else {
            v.push_back(KernelWork{2.0 * a2 * K * C * P, 4.0 * a2 * (K * C + C * P) + out_b});
        }
        return v;
    }
    const double direct = 2.0 * N * K * C * Ho * Wo * L.s.kh * L.s.kw;
    if (s.kind == MNN_SCHEME_GEMM1X1 && s.variant > 0) {
        // Strassen: per level an expand and a combine pass over 7/4 of the operands, 7/8 of the products
        double flops = direct, bb = in_b, pb = out_b;
        for (int l = 0; l < s.variant; ++l) {
            v.push_back(KernelWork{0.0, bb + 1.75 * bb});
            v.push_back(KernelWork{0.0, 1.75 * pb + pb});
            flops *= 0.875; bb *= 1.75; pb *= 1.75;
        }
        v.push_back(KernelWork{flops, bb + pb + w_b});
        return v;
    }
    v.push_back(KernelWork{direct, in_b + out_b + w_b});
    return v;
}

double predict_ms(const Layer& L, const mnn_scheme& s)
{
    mnn_device_model m;
    {
        std::lock_guard<std::mutex> lk(g_model_mu);
        m = g_model;
    }
    // bf16x3 runs three bf16 products per fp32 one at 16x the fp32 matrix-core rate; plain bf16 one
    const double rate = s.prec == MNN_GEMM_BF16X3 ? m.flops * 16.0 / 3.0 : s.prec == MNN_GEMM_BF16 ? m.flops * 16.0 : m.flops;
    double ms = 0.0;
    for (const KernelWork& k : scheme_kernels(L, s))
        ms += std::max(k.flops / rate, k.bytes / m.bytes_per_s) * 1e3 + m.t_schedule_ms;
    return ms;
}

int select_scheme(const mnn_scheme* c, int count, int k)
{
    int best = -1;
    for (int i = 0; i < count; ++i)
        if (c[i].est_ms >= 0.f && (best < 0 || c[i].est_ms < c[best].est_ms)) best = i;
    if (best < 0) return -1;
    const float limit = c[best].est_ms * 1.02f;
    auto alpha_of = [k](const mnn_scheme& s) { return s.kind == MNN_SCHEME_WINOGRAD ? s.tile_n + k - 1 : k; };
    int pick = -1;
    for (int i = 0; i < count; ++i) {
        if (c[i].est_ms < 0.f || c[i].est_ms > limit) continue;
        if (pick < 0) { pick = i; continue; }
        const auto ki = std::make_tuple(alpha_of(c[i]), c[i].prec, c[i].est_ms, c[i].variant);
        const auto kp = std::make_tuple(alpha_of(c[pick]), c[pick].prec, c[pick].est_ms, c[pick].variant);
        if (ki < kp) pick = i;
    }
    return pick;
}

// ------------------------------------------------------------------ GEMM tile configuration per shape
// The matrix-multiplication stage has several tile configurations; which one is fastest depends on
// the shape (how many tiles there are to fill 256 CUs, how long the reduction is).  Like the scheme
// itself it is chosen by measurement at pre-inference time and remembered per shape.
using GemmKey = std::tuple<int, std::vector<long long>>;
std::mutex g_gemm_mu;
struct GemmChoice { int variant; int splitk; };
std::map<GemmKey, GemmChoice> g_gemm_choice;

GemmKey gemm_key(int device, const GemmProblem& p)
{
    std::vector<long long> v = {p.M, p.Ncols, p.R, p.batch, p.lda, p.L, p.strideA_batch, p.strideB_batch, p.strideB_img,
                                p.strideB_row, p.strideD_batch, p.strideD_img, p.strideD_row, p.bias ? 1 : 0,
                                p.gather, p.cv_C, p.cv_H, p.cv_W, p.cv_kh, p.cv_kw, p.cv_sh, p.cv_sw, p.cv_ph, p.cv_pw,
                                p.cv_dh, p.cv_dw, p.cv_Wo, p.prec};
    return GemmKey(device, v);
}

// Times one configuration (warm-up + `iters` launches between two events); *ms < 0 when it does not apply.
int time_gemm(const GemmProblem& p, hipStream_t s, hipEvent_t e0, hipEvent_t e1, int iters, float* ms)
{
    *ms = -1.f;
    hipError_t e = launch_gemm_f32(p, s);
    if (e == hipErrorInvalidValue) { (void)hipGetLastError(); return MNN_OK; }
    if (e != hipSuccess) return fail_hip(e, "gemm tuning launch");
    if ((e = hipEventRecord(e0, s)) != hipSuccess) return fail_hip(e, "hipEventRecord");
    for (int i = 0; i < iters && e == hipSuccess; ++i) e = launch_gemm_f32(p, s);
    if (e != hipSuccess) return fail_hip(e, "gemm tuning launch");
    if ((e = hipEventRecord(e1, s)) != hipSuccess) return fail_hip(e, "hipEventRecord");
    if ((e = hipEventSynchronize(e1)) != hipSuccess) return fail_hip(e, "hipEventSynchronize");
    if ((e = hipEventElapsedTime(ms, e0, e1)) != hipSuccess) return fail_hip(e, "hipEventElapsedTime");
    return MNN_OK;
}

bool cached_gemm_choice(const GemmProblem& p, GemmChoice* out)
{
    int dev = 0;
    (void)hipGetDevice(&dev);
    std::lock_guard<std::mutex> lk(g_gemm_mu);
    auto it = g_gemm_choice.find(gemm_key(dev, p));
    if (it == g_gemm_choice.end()) return false;
    *out = it->second;
    return true;
}

// Times every usable tile configuration -- and, where the tiles do not fill the chip, every useful
// split of the reduction -- on the given (valid, writable) buffers; returns the fastest.
int tune_gemm(GemmProblem p, hipStream_t s, GemmChoice* out)
{
    int dev = 0;
    (void)hipGetDevice(&dev);
    const GemmKey key = gemm_key(dev, p);
    {
        std::lock_guard<std::mutex> lk(g_gemm_mu);
        auto it = g_gemm_choice.find(key);
        if (it != g_gemm_choice.end()) { *out = it->second; return MNN_OK; }
    }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e;
    if ((e = hipEventCreate(&e0)) != hipSuccess) return fail_hip(e, "hipEventCreate");
    if ((e = hipEventCreate(&e1)) != hipSuccess) { (void)hipEventDestroy(e0); return fail_hip(e, "hipEventCreate"); }
    GemmChoice best{0, 1};
    float best_ms = -1.f;
    const int iters = 4;
    int rc = MNN_OK;
    const bool tune_log = std::getenv("MNNCONV_TUNE_LOG") != nullptr;    // one line per timed configuration on stderr
    for (int v = 1; v < gemm_variant_count(p.prec) && !rc; ++v) {
        p.variant = v;
        p.splitk = 1; p.splitk_partial = nullptr;
        float ms = -1.f;
        if ((rc = time_gemm(p, s, e0, e1, iters, &ms))) break;
        if (ms >= 0.f && (best_ms < 0.f || ms < best_ms)) { best_ms = ms; best = GemmChoice{v, 1}; }
        if (tune_log && ms >= 0.f)
            std::fprintf(stderr, "[mnnconv tune] M=%d cols=%d R=%d batch=%d gather=%d %s: %.2f us\n", p.M, p.Ncols, p.R, p.batch,
                         p.gather, gemm_variant_name(p.prec, v), ms * 1e3f / iters);
        int bm = 0, bn = 0, bk = 0;
        if (ms < 0.f || !gemm_variant_tile(p.prec, v, &bm, &bn, &bk)) continue;
        const long long tiles = (long long)((p.M + bm - 1) / bm) * ((p.Ncols + bn - 1) / bn) * p.batch;
        const int chunks = (p.R + bk - 1) / bk;
        // every split count whose slices are all non-empty and equally long up to the last one:
        // sk = ceil(chunks / per) for per = chunks/2 ... 1 chunks per slice
        int prev_sk = 1;
        for (int per = chunks / 2; per >= 1 && !rc; --per) {
            const int sk = (chunks + per - 1) / per;
            if (sk == prev_sk) continue;
            prev_sk = sk;
            if (tiles >= 512 || tiles * sk > 2048 || sk > 64) break;
            const long long pf = gemm_splitk_workspace(p, sk);
            float* part = nullptr;
            if ((e = hipMalloc((void**)&part, (size_t)pf * sizeof(float))) != hipSuccess) {
                rc = fail_hip(e, "hipMalloc split-K scratch");
                break;
            }
            p.splitk = sk; p.splitk_partial = part;
            rc = time_gemm(p, s, e0, e1, iters, &ms);
            (void)hipFree(part);
            if (!rc && ms >= 0.f && ms < best_ms) { best_ms = ms; best = GemmChoice{v, sk}; }
            if (tune_log && !rc && ms >= 0.f)
                std::fprintf(stderr, "[mnnconv tune]     %s splitk=%d: %.2f us\n", gemm_variant_name(p.prec, v), sk, ms * 1e3f / iters);
        }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    *out = best;
    std::lock_guard<std::mutex> lk(g_gemm_mu);
    g_gemm_choice[key] = best;
    return MNN_OK;
}

// ------------------------------------------------------------------ Strassen (Section 3.3.2)
struct Strassen {
    GemmProblem top{};                    // the caller's problem (pointers filled per call), batch 1
    int levels = 0;
    std::vector<float*> Ax, Bx, Px;       // index l = 1..levels: [7^l][R_l][M_l], [7^l][R_l][N_l], [7^l][M_l][N_l]
    GemmChoice choice{0, 1};
    float* sk_partial = nullptr;
    size_t bytes = 0;
    bool left_set = false;

    ~Strassen()
    {
        for (float* q : Ax) if (q) (void)hipFree(q);
        for (float* q : Bx) if (q) (void)hipFree(q);
        for (float* q : Px) if (q) (void)hipFree(q);
        if (sk_partial) (void)hipFree(sk_partial);
    }

    static long long pow7(int l) { long long v = 1; while (l-- > 0) v *= 7; return v; }
    int Ml(int l) const { return top.M >> l; }
    int Rl(int l) const { return top.R >> l; }
    int Nl(int l) const { return top.Ncols >> l; }

    GemmProblem leaf_problem() const
    {
        const int L = levels;
        GemmProblem p{};
        p.At = Ax[L]; p.B = Bx[L]; p.D = Px[L]; p.bias = nullptr;
        p.M = Ml(L); p.Ncols = Nl(L); p.R = Rl(L); p.batch = (int)pow7(L);
        p.lda = Ml(L); p.L = Nl(L);
        p.strideA_batch = (long long)Rl(L) * Ml(L);
        p.strideB_batch = (long long)Rl(L) * Nl(L); p.strideB_img = 0; p.strideB_row = Nl(L);
        p.strideD_batch = (long long)Ml(L) * Nl(L); p.strideD_img = 0; p.strideD_row = Nl(L);
        p.variant = choice.variant; p.prec = top.prec;
        p.splitk = choice.splitk > 1 ? choice.splitk : 1;
        p.splitk_partial = sk_partial;
        return p;
    }

    int init(const GemmProblem& problem, int want_levels, hipStream_t s)
    {
        top = problem;
        if (top.batch != 1) return fail(MNN_E_INVALID_ARG, "Strassen takes one matrix product (batch 1)");
        if (want_levels < 0 || want_levels > 4) return fail(MNN_E_INVALID_ARG, "levels must be 0..4");
        if (want_levels > 0) {
            const int div = 4 << want_levels;
            if (top.M % div || top.Ncols % div || top.R % (1 << want_levels))
                return fail(MNN_E_UNSUPPORTED, "%d Strassen levels need M and ncols divisible by %d and R by %d", want_levels, div,
                            1 << want_levels);
            if (top.L % 4 || top.lda % 4 || top.strideB_img % 4 || top.strideB_row % 4 || top.strideD_img % 4 || top.strideD_row % 4)
                return fail(MNN_E_UNSUPPORTED, "Strassen needs L, lda and all strides divisible by 4");
            if (pow7(want_levels) * top.M >= (1ll << 31)) return fail(MNN_E_UNSUPPORTED, "too many sub-products");
        }
        levels = want_levels;
        Ax.assign(levels + 1, nullptr); Bx.assign(levels + 1, nullptr); Px.assign(levels + 1, nullptr);
        hipError_t e;
        for (int l = 1; l <= levels; ++l) {
            const size_t nb = (size_t)pow7(l);
            const size_t ab = nb * Rl(l) * Ml(l) * sizeof(float), bb = nb * Rl(l) * Nl(l) * sizeof(float),
                         pb = nb * Ml(l) * Nl(l) * sizeof(float);
            if ((e = hipMalloc((void**)&Ax[l], ab)) != hipSuccess || (e = hipMalloc((void**)&Bx[l], bb)) != hipSuccess ||
                (e = hipMalloc((void**)&Px[l], pb)) != hipSuccess)
                return fail_hip(e, "hipMalloc Strassen operands");
            bytes += ab + bb + pb;
        }
        if (levels == 0) {
            // the plain product: tile configuration by timing on scratch operands of the caller's extents
            const long long imgs = (top.Ncols + top.L - 1) / top.L;
            const size_t ab = (size_t)top.R * top.lda * sizeof(float);
            const size_t bb = (size_t)((imgs - 1) * top.strideB_img + (long long)(top.R - 1) * top.strideB_row + top.L) * sizeof(float);
            const size_t db = (size_t)((imgs - 1) * top.strideD_img + (long long)(top.M - 1) * top.strideD_row + top.L) * sizeof(float);
            float *ta = nullptr, *tb = nullptr, *td = nullptr;
            int rc = MNN_OK;
            if ((e = hipMalloc((void**)&ta, ab)) != hipSuccess || (e = hipMalloc((void**)&tb, bb)) != hipSuccess ||
                (e = hipMalloc((void**)&td, db)) != hipSuccess || (e = hipMemset(ta, 0, ab)) != hipSuccess ||
                (e = hipMemset(tb, 0, bb)) != hipSuccess)
                rc = fail_hip(e, "Strassen tuning scratch");
            if (!rc) {
                GemmProblem p = top;
                p.At = ta; p.B = tb; p.D = td; p.bias = nullptr; p.variant = 0; p.splitk = 1; p.splitk_partial = nullptr;
                rc = tune_gemm(p, s, &choice);
                if (!rc && choice.splitk > 1) {
                    const size_t pb = (size_t)gemm_splitk_workspace(p, choice.splitk) * sizeof(float);
                    if ((e = hipMalloc((void**)&sk_partial, pb)) != hipSuccess) rc = fail_hip(e, "hipMalloc split-K partials");
                    bytes += pb;
                }
            }
            if (ta) (void)hipFree(ta);
            if (tb) (void)hipFree(tb);
            if (td) (void)hipFree(td);
            if (rc) return rc;
            top.variant = choice.variant;
            top.splitk = choice.splitk > 1 ? choice.splitk : 1;
            top.splitk_partial = sk_partial;
        }
        if (levels > 0) {
            // tile configuration of the one batched GEMM at the bottom, by timing like any other shape
            GemmProblem p = leaf_problem();
            p.variant = 0; p.splitk = 1; p.splitk_partial = nullptr;
            int rc = tune_gemm(p, s, &choice);
            if (rc) return rc;
            if (choice.splitk > 1) {
                const size_t pb = (size_t)gemm_splitk_workspace(p, choice.splitk) * sizeof(float);
                if ((e = hipMalloc((void**)&sk_partial, pb)) != hipSuccess) return fail_hip(e, "hipMalloc split-K partials");
                bytes += pb;
            }
        }
        return MNN_OK;
    }

    // expands the left operand (weights) for all levels; once per weight set
    int set_left(const float* At, hipStream_t s)
    {
        if (!At) return fail(MNN_E_INVALID_ARG, "At is NULL");
        top.At = At;
        hipError_t e = hipSuccess;
        for (int l = 1; l <= levels && e == hipSuccess; ++l) {
            const StrassenView v = (l == 1) ? StrassenView{top.lda, 0, top.lda} : StrassenView{Ml(l - 1), 0, Ml(l - 1)};
            const float* src = (l == 1) ? At : Ax[l - 1];
            const long long sb = (l == 1) ? 0 : (long long)Rl(l - 1) * Ml(l - 1);
            e = launch_strassen_expand(true, v, src, sb, Rl(l), Ml(l), (int)pow7(l - 1), Ax[l], s);
        }
        if (e != hipSuccess) return fail_hip(e, "Strassen left expansion");
        left_set = true;
        return MNN_OK;
    }

    int run(const float* B, const float* bias, float* D, hipStream_t s)
    {
        if (!B || !D) return fail(MNN_E_INVALID_ARG, "B and D must not be NULL");
        if (!left_set) return fail(MNN_E_INVALID_ARG, "the left operand has not been set");
        hipError_t e = hipSuccess;
        if (levels == 0) {
            GemmProblem p = top;
            p.B = B; p.D = D; p.bias = bias;
            e = launch_gemm_f32(p, s);
            if (e != hipSuccess) return fail_hip(e, "gemm launch");
            return MNN_OK;
        }
        for (int l = 1; l <= levels && e == hipSuccess; ++l) {
            const StrassenView v = (l == 1) ? StrassenView{top.L, top.strideB_img, top.strideB_row} : StrassenView{Nl(l - 1), 0, Nl(l - 1)};
            const float* src = (l == 1) ? B : Bx[l - 1];
            const long long sb = (l == 1) ? 0 : (long long)Rl(l - 1) * Nl(l - 1);
            e = launch_strassen_expand(false, v, src, sb, Rl(l), Nl(l), (int)pow7(l - 1), Bx[l], s);
        }
        if (e == hipSuccess) e = launch_gemm_f32(leaf_problem(), s);
        for (int l = levels; l >= 1 && e == hipSuccess; --l) {
            const StrassenView v = (l == 1) ? StrassenView{top.L, top.strideD_img, top.strideD_row} : StrassenView{Nl(l - 1), 0, Nl(l - 1)};
            float* dst = (l == 1) ? D : Px[l - 1];
            const long long db = (l == 1) ? 0 : (long long)Ml(l - 1) * Nl(l - 1);
            e = launch_strassen_combine(v, Px[l], Ml(l), Nl(l), (int)pow7(l - 1), dst, db, l == 1 ? bias : nullptr, s);
        }
        if (e != hipSuccess) return fail_hip(e, "Strassen launch");
        return MNN_OK;
    }

    int launches() const { return 2 * levels + 1 + (choice.splitk > 1 ? 1 : 0); }
};

// ------------------------------------------------------------------ one realised scheme
struct Impl {
    mnn_scheme scheme{};
    Layer L{};
    WinogradMatrices mats;      // along H (both axes of a square kernel)
    WinogradMatrices mats_w;    // along W (kernels with one row or column; the untransformed axis holds 1 x 1 identities)
    bool rect = false;
    std::unique_ptr<Strassen> strassen;   // 1x1 scheme with scheme.variant = Strassen levels > 0
    WinoGeom wg{};
    float* U = nullptr; size_t U_bytes = 0;
    float* V = nullptr; size_t V_bytes = 0;
    float* M = nullptr; size_t M_bytes = 0;
    int ldk = 0;
    int gemm_variant = 0;      // tile configuration of the GEMM stage (0 = shape heuristic)
    int gemm_splitk = 1;       // workgroups per tile along the reduction
    float* sk_partial = nullptr; size_t sk_partial_bytes = 0;
    // V, M and the split-K partials hold nothing between two runs.  A plan on its own allocates them;
    // a chain of layers binds them to a region of its arena instead (bind_transient).
    bool transient_external = false;

    ~Impl() { release(); }
    Impl() = default;
    Impl(const Impl&) = delete;
    Impl& operator=(const Impl&) = delete;

    void release()
    {
        if (U) (void)hipFree(U);
        if (!transient_external) {
            if (V) (void)hipFree(V);
            if (M) (void)hipFree(M);
            if (sk_partial) (void)hipFree(sk_partial);
        }
        U = V = M = nullptr;
        sk_partial = nullptr;
        U_bytes = V_bytes = M_bytes = sk_partial_bytes = 0;
    }

    int alloc_zero(float** p, size_t bytes, const char* what)
    {
        hipError_t e = hipMalloc((void**)p, bytes);
        if (e != hipSuccess) { *p = nullptr; return fail_hip(e, what); }
        e = hipMemset(*p, 0, bytes);
        if (e != hipSuccess) return fail_hip(e, what);
        // plan time: make the cleared padding visible to whatever stream runs the plan later
        e = hipDeviceSynchronize();
        if (e != hipSuccess) return fail_hip(e, what);
        return MNN_OK;
    }

    int alloc_transient(float** p, size_t bytes, const char* what)
    {
        if (transient_external) { *p = nullptr; return MNN_OK; }
        return alloc_zero(p, bytes, what);
    }

    static size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }
    size_t transient_bytes() const { return align256(V_bytes) + align256(M_bytes) + align256(sk_partial_bytes); }
    void bind_transient(char* base)
    {
        V = V_bytes ? reinterpret_cast<float*>(base) : nullptr;
        M = M_bytes ? reinterpret_cast<float*>(base + align256(V_bytes)) : nullptr;
        sk_partial = sk_partial_bytes ? reinterpret_cast<float*>(base + align256(V_bytes) + align256(M_bytes)) : nullptr;
    }

    int prepare(const Layer& layer, const mnn_scheme& s, const mnn_conv_options& o, bool external_transient = false)
    {
        L = layer;
        scheme = s;
        transient_external = external_transient;
        const mnn_conv_shape& sh = L.s;
        ldk = round_up(sh.c_out, 4);
        if (s.prec != MNN_GEMM_FP32 && s.kind == MNN_SCHEME_WINOGRAD && s.variant != MNN_WINO_UNFUSED)
            return fail(MNN_E_UNSUPPORTED, "the fused Winograd kernels multiply in fp32 only");
        if (s.kind == MNN_SCHEME_WINOGRAD) {
            if (!winograd_admissible(L))
                return fail(MNN_E_UNSUPPORTED, "Winograd needs a square kernel >= 2 (or 1 x k / k x 1), stride 1, dilation 1");
            rect = winograd_rect(L);
            const int n = s.tile_n, k = wino_k(L);
            if (!winograd_kernels_available(n, k))
                return fail(MNN_E_UNSUPPORTED, "F(%d,%d) is outside the built range (n 2..8, k 2..7, alpha <= %d)", n, k, kMaxAlphaT);
            WinogradMatrices gen, unit;
            // f = 0: the scale with the least fp32 error for this alpha.  Up to alpha = 8 that is the paper's 0.5;
            // for 9 and 10 points spaced 0.425 apart bring the error down 3-5x (points further out blow up G, points
            // closer together blow up B^T).
            const double f = o.point_scale_f > 0.f ? (double)o.point_scale_f : (n + k - 1 >= 9 ? 0.425 : 0.5);
            if (!generate_winograd(n, k, f, &gen))
                return fail(MNN_E_UNSUPPORTED, "generator rejected F(%d,%d)", n, k);
            unit.n = unit.k = unit.alpha = 1;
            unit.AT.assign(1, 1.f); unit.G.assign(1, 1.f); unit.BT.assign(1, 1.f);
            mats = (rect && sh.kh == 1) ? unit : gen;
            mats_w = (rect && sh.kw == 1) ? unit : gen;
            wg.N = sh.n; wg.C = sh.c_in; wg.H = sh.h; wg.W = sh.w; wg.K = sh.c_out;
            wg.Ho = L.Ho; wg.Wo = L.Wo; wg.pad_h = L.g.pad_h; wg.pad_w = L.g.pad_w;
            wg.n = mats.n; wg.k = mats.k; wg.alpha = mats.alpha;
            wg.nw = mats_w.n; wg.kw = mats_w.k; wg.alpha_w = mats_w.alpha;
            wg.th = (L.Ho + wg.n - 1) / wg.n; wg.tw = (L.Wo + wg.nw - 1) / wg.nw;
            const long long P = (long long)sh.n * wg.th * wg.tw;
            if (P >= (1ll << 30)) return fail(MNN_E_UNSUPPORTED, "too many tiles");
            wg.P = (int)P; wg.ldp = round_up(wg.P, 4); wg.ldk = ldk;
            const size_t a2 = (size_t)wg.alpha * wg.alpha_w;
            if (rect && s.variant != MNN_WINO_UNFUSED)
                return fail(MNN_E_UNSUPPORTED, "kernels with one row or column have no fused variant");
            if (!wino_variant_available(n, k, s.variant))
                return fail(MNN_E_UNSUPPORTED, "Winograd variant %d is not available for F(%d,%d)", s.variant, n, k);
            int rc;
            if (s.variant != MNN_WINO_UNFUSED) {
                // blocked operands, padded so that whole 128-wide blocks can be copied unchecked
                wg.blocked = 1;
                wg.cchunks = round_up((sh.c_in + 3) / 4, 4);          // whole 16-channel chunks
                wg.kg = round_up((sh.c_out + 15) / 16, 8);
                wg.pg = round_up((wg.P + 15) / 16, 8);
                U_bytes = (size_t)wg.cchunks * a2 * wg.kg * 64 * sizeof(float);
                V_bytes = (size_t)wg.cchunks * a2 * wg.pg * 64 * sizeof(float);
                if (V_bytes >= ((size_t)1 << 40) || U_bytes >= ((size_t)1 << 40))
                    return fail(MNN_E_UNSUPPORTED, "Winograd-domain tensors too large");
                if ((rc = alloc_zero(&U, U_bytes, "hipMalloc U"))) return rc;
                if ((rc = alloc_transient(&V, V_bytes, "hipMalloc V"))) return rc;
                return MNN_OK;
            }
            if ((long long)wg.C * wg.ldp >= (1ll << 31) || (long long)wg.K * wg.ldp >= (1ll << 31))
                return fail(MNN_E_UNSUPPORTED, "Winograd-domain plane too large");
            U_bytes = a2 * sh.c_in * ldk * sizeof(float);
            V_bytes = a2 * sh.c_in * wg.ldp * sizeof(float);
            M_bytes = a2 * sh.c_out * wg.ldp * sizeof(float);
            if ((rc = alloc_zero(&U, U_bytes, "hipMalloc U"))) return rc;
            if ((rc = alloc_transient(&V, V_bytes, "hipMalloc V"))) return rc;
            if ((rc = alloc_transient(&M, M_bytes, "hipMalloc M"))) return rc;
            return MNN_OK;
        }
        if (s.kind == MNN_SCHEME_GEMM1X1) {
            if (!is_pointwise(L)) return fail(MNN_E_UNSUPPORTED, "GEMM scheme needs a 1x1 kernel, stride 1, no padding");
            if ((long long)sh.n * sh.h * sh.w >= (1ll << 31)) return fail(MNN_E_UNSUPPORTED, "too many pixels");
            U_bytes = (size_t)sh.c_in * ldk * sizeof(float);
            return alloc_zero(&U, U_bytes, "hipMalloc Wt");
        }
        if (s.kind == MNN_SCHEME_DIRECT) {
            // implicit GEMM on the matrix cores: weights transposed to [C*kh*kw][ldk]
            if ((long long)sh.n * L.Ho * L.Wo >= (1ll << 31) || (long long)sh.n * sh.c_in * sh.h * sh.w >= (1ll << 31))
                return fail(MNN_E_UNSUPPORTED, "tensor too large for the sliding-window kernel");
            U_bytes = (size_t)sh.c_in * sh.kh * sh.kw * ldk * sizeof(float);
            int rcd = alloc_zero(&U, U_bytes, "hipMalloc Wt");
            if (rcd) return rcd;
            return MNN_OK;
        }
        return fail(MNN_E_INVALID_ARG, "unknown scheme kind %d", s.kind);
    }

    GemmProblem wino_gemm_problem() const
    {
        GemmProblem p{};
        p.At = U; p.B = V; p.D = M; p.bias = nullptr;
        p.M = wg.K; p.Ncols = wg.ldp; p.R = wg.C; p.batch = wg.alpha * wg.alpha_w;
        p.lda = ldk; p.L = wg.ldp;
        p.strideA_batch = (long long)wg.C * ldk;
        p.strideB_batch = (long long)wg.C * wg.ldp; p.strideB_img = 0; p.strideB_row = wg.ldp;
        p.strideD_batch = (long long)wg.K * wg.ldp; p.strideD_img = 0; p.strideD_row = wg.ldp;
        set_gemm_choice(&p);
        return p;
    }

    void set_gemm_choice(GemmProblem* p) const
    {
        p->variant = gemm_variant;
        p->prec = scheme.prec;
        p->splitk = gemm_splitk;
        p->splitk_partial = sk_partial;
    }

    GemmProblem pointwise_gemm_problem(const float* x, const float* b, float* y) const
    {
        const mnn_conv_shape& sh = L.s;
        const int HW = sh.h * sh.w;
        GemmProblem p{};
        p.At = U; p.B = x; p.D = y; p.bias = b;
        p.M = sh.c_out; p.Ncols = sh.n * HW; p.R = sh.c_in; p.batch = 1;
        p.lda = ldk; p.L = HW;
        p.strideA_batch = 0;
        p.strideB_batch = 0; p.strideB_img = (long long)sh.c_in * HW; p.strideB_row = HW;
        p.strideD_batch = 0; p.strideD_img = (long long)sh.c_out * HW; p.strideD_row = HW;
        set_gemm_choice(&p);
        return p;
    }

    GemmProblem direct_gemm_problem(const float* x, const float* b, float* y) const
    {
        const mnn_conv_shape& sh = L.s;
        const int HoWo = L.Ho * L.Wo;
        GemmProblem p{};
        p.At = U; p.B = x; p.D = y; p.bias = b;
        p.M = sh.c_out; p.Ncols = sh.n * HoWo; p.R = sh.c_in * sh.kh * sh.kw; p.batch = 1;
        p.lda = ldk; p.L = HoWo;
        p.strideD_img = (long long)sh.c_out * HoWo; p.strideD_row = HoWo;
        set_gemm_choice(&p);
        p.gather = 1;
        p.cv_C = sh.c_in; p.cv_H = sh.h; p.cv_W = sh.w; p.cv_kh = sh.kh; p.cv_kw = sh.kw;
        p.cv_sh = L.g.stride_h; p.cv_sw = L.g.stride_w; p.cv_ph = L.g.pad_h; p.cv_pw = L.g.pad_w;
        p.cv_dh = L.g.dil_h; p.cv_dw = L.g.dil_w; p.cv_Wo = L.Wo;
        return p;
    }

    // Picks the GEMM tile configuration by timing (pre-inference).  The 1x1 scheme multiplies the
    // caller's tensors, so it is tuned on scratch tensors of the layer's size.
    int adopt(const GemmProblem& p, const GemmChoice& c)
    {
        gemm_variant = c.variant;
        gemm_splitk = c.splitk > 1 ? c.splitk : 1;
        if (gemm_splitk == 1) return MNN_OK;
        int bm = 0, bn = 0, bk = 0;
        if (!gemm_variant_tile(p.prec, gemm_variant, &bm, &bn, &bk)) { gemm_splitk = 1; return MNN_OK; }
        sk_partial_bytes = (size_t)gemm_splitk_workspace(p, gemm_splitk) * sizeof(float);
        return alloc_transient(&sk_partial, sk_partial_bytes, "hipMalloc split-K partials");
    }

    int tune(hipStream_t s)
    {
        GemmChoice c{0, 1};
        static const float dummy_bias = 0.f;      // only "is there a bias" enters the cache key
        if (scheme.kind == MNN_SCHEME_WINOGRAD && scheme.variant == MNN_WINO_UNFUSED) {
            const GemmProblem p = wino_gemm_problem();
            if (transient_external) {
                // V and M are not bound yet: take the remembered choice, else the shape heuristic
                if (!cached_gemm_choice(p, &c)) c = GemmChoice{0, 1};
                return adopt(p, c);
            }
            int rc = tune_gemm(p, s, &c);
            return rc ? rc : adopt(p, c);
        }
        if (scheme.kind == MNN_SCHEME_GEMM1X1 && scheme.variant > 0) {
            if (scheme.prec != MNN_GEMM_FP32) return fail(MNN_E_UNSUPPORTED, "Strassen runs on the fp32 GEMM only");
            strassen.reset(new Strassen());
            GemmProblem p = pointwise_gemm_problem(nullptr, nullptr, nullptr);
            p.variant = 0; p.splitk = 1; p.splitk_partial = nullptr;
            return strassen->init(p, scheme.variant, s);
        }
        if (scheme.kind == MNN_SCHEME_GEMM1X1 || scheme.kind == MNN_SCHEME_DIRECT) {
            const mnn_conv_shape& sh = L.s;
            const size_t xb = (size_t)sh.n * sh.c_in * sh.h * sh.w * sizeof(float);
            const size_t yb = (size_t)sh.n * sh.c_out * L.Ho * L.Wo * sizeof(float);
            float *tx = nullptr, *ty = nullptr, *tb = nullptr;
            hipError_t e;
            int rc = MNN_OK;
            {
                // a shape tuned before needs no scratch tensors (the key holds no addresses)
                const GemmProblem q = scheme.kind == MNN_SCHEME_DIRECT ? direct_gemm_problem(nullptr, &dummy_bias, nullptr)
                                                                       : pointwise_gemm_problem(nullptr, &dummy_bias, nullptr);
                if (cached_gemm_choice(q, &c)) return adopt(q, c);
            }
            if ((e = hipMalloc((void**)&tx, xb)) != hipSuccess || (e = hipMalloc((void**)&ty, yb)) != hipSuccess ||
                (e = hipMalloc((void**)&tb, (size_t)sh.c_out * sizeof(float))) != hipSuccess)
                rc = fail_hip(e, "hipMalloc tuning scratch");
            if (!rc && ((e = hipMemset(tx, 0, xb)) != hipSuccess || (e = hipMemset(tb, 0, (size_t)sh.c_out * sizeof(float))) != hipSuccess))
                rc = fail_hip(e, "hipMemset tuning scratch");
            GemmProblem p = scheme.kind == MNN_SCHEME_DIRECT ? direct_gemm_problem(tx, tb, ty) : pointwise_gemm_problem(tx, tb, ty);
            if (!rc) rc = tune_gemm(p, s, &c);
            if (tx) (void)hipFree(tx);
            if (ty) (void)hipFree(ty);
            if (tb) (void)hipFree(tb);
            return rc ? rc : adopt(p, c);
        }
        return MNN_OK;
    }

    bool has_stage(int st) const
    {
        switch (scheme.kind) {
            case MNN_SCHEME_WINOGRAD: return scheme.variant == MNN_WINO_UNFUSED || st != MNN_STAGE_OUTPUT;
            case MNN_SCHEME_GEMM1X1: return st == MNN_STAGE_FILTER || st == MNN_STAGE_GEMM;
            default: return st == MNN_STAGE_FILTER || st == MNN_STAGE_GEMM;
        }
    }

    int run_stage(int st, const float* x, const float* w, const float* b, float* y, hipStream_t s)
    {
        if (!has_stage(st)) return MNN_OK;
        hipError_t e = hipSuccess;
        const mnn_conv_shape& sh = L.s;
        if (scheme.kind == MNN_SCHEME_WINOGRAD) {
            switch (st) {
                case MNN_STAGE_FILTER:
                    e = rect ? launch_filter_transform_rect(wg, mats.G.data(), mats_w.G.data(), w, U, s)
                             : launch_filter_transform(wg, mats.G.data(), w, U, s);
                    break;
                case MNN_STAGE_INPUT:
                    e = rect ? launch_input_transform_rect(wg, mats.BT.data(), mats_w.BT.data(), x, V, s)
                             : launch_input_transform(wg, mats.BT.data(), x, V, s);
                    break;
                case MNN_STAGE_GEMM: {
                    if (scheme.variant != MNN_WINO_UNFUSED) {
                        e = launch_wino_fused(wg, scheme.variant - 1, mats.AT.data(), U, V, b, y, s);
                        break;
                    }
                    e = launch_gemm_f32(wino_gemm_problem(), s);
                    break;
                }
                case MNN_STAGE_OUTPUT:
                    e = rect ? launch_output_transform_rect(wg, mats.AT.data(), mats_w.AT.data(), M, b, y, s)
                             : launch_output_transform(wg, mats.AT.data(), M, b, y, s);
                    break;
            }
        } else if (scheme.kind == MNN_SCHEME_GEMM1X1) {
            const int HW = sh.h * sh.w;
            if (st == MNN_STAGE_FILTER) {
                e = launch_weight_transpose(w, U, sh.c_out, sh.c_in, ldk, s);
                if (e == hipSuccess && strassen) {
                    int rc = strassen->set_left(U, s);
                    if (rc) return rc;
                }
            } else if (strassen) {
                return strassen->run(x, b, y, s);
            } else {
                e = launch_gemm_f32(pointwise_gemm_problem(x, b, y), s);
            }
        } else {
            if (st == MNN_STAGE_FILTER)
                e = launch_weight_transpose(w, U, sh.c_out, sh.c_in * sh.kh * sh.kw, ldk, s);
            else
                e = launch_gemm_f32(direct_gemm_problem(x, b, y), s);
        }
        if (e != hipSuccess) return fail_hip(e, "kernel launch");
        return MNN_OK;
    }

    size_t bytes() const { return U_bytes + V_bytes + M_bytes + sk_partial_bytes + (strassen ? strassen->bytes : 0); }
};

void describe_impl(const Impl& im, char* buf, size_t cap)
{
    std::string gvs = gemm_variant_name(im.scheme.prec, im.gemm_variant) ? gemm_variant_name(im.scheme.prec, im.gemm_variant) : "?";
    if (im.gemm_splitk > 1) gvs += " splitk=" + std::to_string(im.gemm_splitk);
    const char* gv = gvs.c_str();
    switch (im.scheme.kind) {
        case MNN_SCHEME_WINOGRAD:
            if (im.rect)
                std::snprintf(buf, cap, "F(%dx%d,%dx%d) unfused gemm=%s", im.wg.n, im.wg.nw, im.wg.k, im.wg.kw, gv);
            else if (im.scheme.variant == MNN_WINO_UNFUSED)
                std::snprintf(buf, cap, "F(%d,%d) unfused gemm=%s", im.wg.n, im.wg.k, gv);
            else
                std::snprintf(buf, cap, "F(%d,%d) fused-output %s", im.wg.n, im.wg.k,
                              im.scheme.variant == MNN_WINO_FUSED_OUT_32 ? "32x32" : "64x64");
            break;
        case MNN_SCHEME_GEMM1X1:
            if (im.strassen) {
                const char* leaf = gemm_variant_name(MNN_GEMM_FP32, im.strassen->choice.variant);
                std::snprintf(buf, cap, "gemm1x1 strassen levels=%d gemm=%s", im.strassen->levels, leaf ? leaf : "?");
            } else {
                std::snprintf(buf, cap, "gemm1x1 gemm=%s", gv);
            }
            break;
        default: std::snprintf(buf, cap, "sliding-window implicit gemm=%s", gv); break;
    }
}

// ------------------------------------------------------------------ choice cache
using CacheKey = std::tuple<int, std::vector<int>, float>;
std::mutex g_cache_mu;
std::map<CacheKey, mnn_scheme> g_cache;

CacheKey cache_key(int device, const Layer& L, const mnn_conv_options& o)
{
    std::vector<int> v = {L.s.n, L.s.c_in, L.s.h, L.s.w, L.s.c_out, L.s.kh, L.s.kw,
                          L.g.stride_h, L.g.stride_w, L.g.pad_h, L.g.pad_w, L.g.dil_h, L.g.dil_w,
                          o.alpha_max, o.allow_bf16, (int)std::lround((double)o.prune_ratio * 1000.0)};
    return CacheKey(device, v, o.point_scale_f);
}

}  // namespace

struct mnn_conv_plan_s {
    Layer L{};
    mnn_conv_options opt{};
    int device = 0;
    Impl impl;
    std::vector<mnn_scheme> cands;
    const float* cached_weight = nullptr;
    bool weights_valid = false;
    bool from_cache = false;
};


struct mnn_chain_s {
    std::vector<Layer> layers;
    mnn_conv_options opt{};
    int device = 0;
    std::vector<std::unique_ptr<Impl>> impls;
    std::vector<float*> bias;            // chain-owned copies (c_out floats each)
    std::vector<char> has_bias, weights_set;
    char* arena = nullptr;
    size_t arena_bytes = 0, unshared_bytes = 0, live_peak_bytes = 0, weight_bytes = 0;
    std::vector<long long> act_off, ws_off;     // activation i = output of layer i (i < n-1); workspace of layer i
    std::vector<size_t> act_bytes;
    hipStream_t capture_stream = nullptr;
    hipGraph_t graph = nullptr;
    hipGraphExec_t exec = nullptr;
    size_t graph_nodes = 0;

    ~mnn_chain_s()
    {
        if (exec) (void)hipGraphExecDestroy(exec);
        if (graph) (void)hipGraphDestroy(graph);
        if (capture_stream) (void)hipStreamDestroy(capture_stream);
        impls.clear();
        for (float* b : bias)
            if (b) (void)hipFree(b);
        if (arena) (void)hipFree(arena);
    }

    int kernels_per_run() const
    {
        int k = 0;
        for (const auto& im : impls)
            for (int st = MNN_STAGE_INPUT; st < MNN_STAGE_COUNT; ++st)
                if (im->has_stage(st))
                    k += (st == MNN_STAGE_GEMM && im->strassen) ? im->strassen->launches()
                         : (st == MNN_STAGE_GEMM && im->gemm_splitk > 1) ? 2 : 1;                // + the slice reduction
        return k;
    }

    int enqueue(const float* input, float* output, hipStream_t s)
    {
        const int n = (int)impls.size();
        for (int i = 0; i < n; ++i) {
            const float* x = i == 0 ? input : reinterpret_cast<const float*>(arena + act_off[i - 1]);
            float* y = i == n - 1 ? output : reinterpret_cast<float*>(arena + act_off[i]);
            const float* b = has_bias[i] ? bias[i] : nullptr;
            for (int st = MNN_STAGE_INPUT; st < MNN_STAGE_COUNT; ++st) {
                int rc = impls[i]->run_stage(st, x, nullptr, b, y, s);
                if (rc) return rc;
            }
        }
        return MNN_OK;
    }
};

namespace {

struct Scratch {
    float *x = nullptr, *w = nullptr, *y = nullptr;
    ~Scratch()
    {
        if (x) (void)hipFree(x);
        if (w) (void)hipFree(w);
        if (y) (void)hipFree(y);
    }
};

// Times one candidate: `warmup` untimed and `iters` timed passes of the
// per-inference stages, bracketed by HIP events on `s`.
int time_candidate(const Layer& L, const mnn_conv_options& o, mnn_scheme* cand, const Scratch& sc, hipStream_t s)
{
    Impl impl;
    int rc = impl.prepare(L, *cand, o);
    if (rc) return rc;
    if ((rc = impl.tune(s))) return rc;
    if ((rc = impl.run_stage(MNN_STAGE_FILTER, sc.x, sc.w, nullptr, sc.y, s))) return rc;
    auto pass = [&]() -> int {
        for (int st = MNN_STAGE_INPUT; st < MNN_STAGE_COUNT; ++st) {
            int r = impl.run_stage(st, sc.x, sc.w, nullptr, sc.y, s);
            if (r) return r;
        }
        return MNN_OK;
    };
    for (int i = 0; i < o.plan_warmup; ++i)
        if ((rc = pass())) return rc;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    hipError_t e;
    if ((e = hipEventCreate(&e0)) != hipSuccess) return fail_hip(e, "hipEventCreate");
    if ((e = hipEventCreate(&e1)) != hipSuccess) { (void)hipEventDestroy(e0); return fail_hip(e, "hipEventCreate"); }
    float ms = -1.f;
    rc = MNN_OK;
    do {
        if ((e = hipEventRecord(e0, s)) != hipSuccess) { rc = fail_hip(e, "hipEventRecord"); break; }
        for (int i = 0; i < o.plan_iters && !rc; ++i) rc = pass();
        if (rc) break;
        if ((e = hipEventRecord(e1, s)) != hipSuccess) { rc = fail_hip(e, "hipEventRecord"); break; }
        if ((e = hipEventSynchronize(e1)) != hipSuccess) { rc = fail_hip(e, "hipEventSynchronize"); break; }
        if ((e = hipEventElapsedTime(&ms, e0, e1)) != hipSuccess) { rc = fail_hip(e, "hipEventElapsedTime"); break; }
    } while (false);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    cand->est_ms = ms / (float)o.plan_iters;
    return MNN_OK;
}

int plan_impl(const mnn_conv_shape* shape, const mnn_conv_geom* geom, const mnn_conv_options* options, void* stream,
              mnn_conv_plan_t* out_plan)
{
    if (!out_plan) return fail(MNN_E_INVALID_ARG, "out_plan must not be NULL");
    Layer L;
    int rc = validate(shape, geom, &L);
    if (rc) return rc;
    mnn_conv_options o;
    if ((rc = validate_options(options, &o))) return rc;

    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        return fail(MNN_E_NO_DEVICE, "no HIP device available (%s)", e == hipSuccess ? "count is 0" : hipGetErrorString(e));
    }
    int dev = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return fail_hip(e, "hipGetDevice");
    hipStream_t s = (hipStream_t)stream;

    mnn_conv_plan_s* plan = new (std::nothrow) mnn_conv_plan_s();
    if (!plan) return fail(MNN_E_OOM, "host allocation failed");
    plan->L = L;
    plan->opt = o;
    plan->device = dev;

    mnn_scheme chosen;
    bool use_cache = o.use_cache != 0;
    if (o.force_kind != MNN_SCHEME_AUTO) {
        use_cache = false;
        if (o.force_kind == MNN_SCHEME_WINOGRAD) {
            int n = o.force_tile_n;
            if (n <= 0) {
                n = analytic_tile(wino_k(L), L.s.c_in, L.s.c_out, L.Ho, L.Wo, o.alpha_max);
                if (n < 2) n = 2;
            }
            if (o.force_variant >= 0)
                plan->cands.push_back(make_scheme(MNN_SCHEME_WINOGRAD, n, o.force_prec, o.force_variant));
            else if (winograd_admissible(L) && winograd_rect(L))
                plan->cands.push_back(make_scheme(MNN_SCHEME_WINOGRAD, n, o.force_prec, MNN_WINO_UNFUSED));
            else if (winograd_admissible(L))
                push_wino_variants(&plan->cands, n, L.s.kh, o.force_prec);   // time the arrangements of this F(n,k)
            if (plan->cands.empty()) plan->cands.push_back(make_scheme(MNN_SCHEME_WINOGRAD, n, o.force_prec, 0));
        } else {
            const int lv = (o.force_kind == MNN_SCHEME_GEMM1X1 && o.force_variant > 0) ? o.force_variant : 0;   // Strassen levels
            plan->cands.push_back(make_scheme(o.force_kind, 0, o.force_prec, lv));
        }
    } else {
        plan->cands = enumerate(L, o);
    }
    {
        bool hit = false;
        const CacheKey key = cache_key(dev, L, o);
        if (use_cache) {
            std::lock_guard<std::mutex> lk(g_cache_mu);
            auto it = g_cache.find(key);
            if (it != g_cache.end()) { chosen = it->second; hit = true; }
        }
        if (!hit) {
            if (plan->cands.size() == 1) {
                chosen = plan->cands[0];
            } else {
                // scratch tensors for the timing launches (contents do not affect kernel time)
                Scratch sc;
                const size_t xb = (size_t)L.s.n * L.s.c_in * L.s.h * L.s.w * sizeof(float);
                const size_t wb = (size_t)L.s.c_out * L.s.c_in * L.s.kh * L.s.kw * sizeof(float);
                const size_t yb = (size_t)L.s.n * L.s.c_out * L.Ho * L.Wo * sizeof(float);
                if ((e = hipMalloc((void**)&sc.x, xb)) != hipSuccess || (e = hipMalloc((void**)&sc.w, wb)) != hipSuccess ||
                    (e = hipMalloc((void**)&sc.y, yb)) != hipSuccess) {
                    delete plan;
                    return fail_hip(e, "hipMalloc planner scratch");
                }
                if ((e = hipMemset(sc.x, 0, xb)) != hipSuccess || (e = hipMemset(sc.w, 0, wb)) != hipSuccess) {
                    delete plan;
                    return fail_hip(e, "hipMemset planner scratch");
                }
                double best_pred = -1.0;
                for (const auto& c : plan->cands) {
                    const double pm = predict_ms(L, c);
                    if (best_pred < 0.0 || pm < best_pred) best_pred = pm;
                }
                for (auto& c : plan->cands) {
                    if (o.prune_ratio > 1.f && predict_ms(L, c) > (double)o.prune_ratio * best_pred) { c.est_ms = -1.f; continue; }
                    rc = time_candidate(L, o, &c, sc, s);
                    if (rc == MNN_E_OOM) { c.est_ms = -1.f; (void)hipGetLastError(); continue; }   // does not fit: not a candidate
                    if (rc) { delete plan; return rc; }
                }
                const int pick = select_scheme(plan->cands.data(), (int)plan->cands.size(), wino_k(L));
                if (pick < 0) { delete plan; return fail(MNN_E_OOM, "no candidate scheme could be timed"); }
                chosen = plan->cands[pick];
            }
            if (use_cache) {
                std::lock_guard<std::mutex> lk(g_cache_mu);
                g_cache[key] = chosen;
            }
        } else {
            plan->from_cache = true;
        }
    }
    rc = plan->impl.prepare(L, chosen, o);
    if (!rc) rc = plan->impl.tune(s);
    if (rc) { delete plan; return rc; }
    *out_plan = plan;
    return MNN_OK;
}

int check_run_args(mnn_conv_plan_t plan, const float* input, const float* weight, float* output)
{
    if (!plan) return fail(MNN_E_INVALID_ARG, "plan is NULL");
    if (!input || !weight || !output) return fail(MNN_E_INVALID_ARG, "input, weight and output must not be NULL");
    return MNN_OK;
}

}  // namespace

extern "C" {

int mnn_conv_options_default(mnn_conv_options* opt)
{
    if (!opt) return fail(MNN_E_INVALID_ARG, "opt is NULL");
    default_options(opt);
    return MNN_OK;
}

int mnn_conv_plan(const mnn_conv_shape* shape, const mnn_conv_geom* geom, const mnn_conv_options* options,
                  void* stream, mnn_conv_plan_t* out_plan)
{
    try {
        return plan_impl(shape, geom, options, stream, out_plan);
    } catch (const std::bad_alloc&) {
        return fail(MNN_E_OOM, "host allocation failed");
    } catch (...) {
        return fail(MNN_E_INVALID_ARG, "unexpected exception in mnn_conv_plan");
    }
}

int mnn_conv_plan_scheme(mnn_conv_plan_t plan, mnn_scheme* out)
{
    if (!plan || !out) return fail(MNN_E_INVALID_ARG, "NULL argument");
    *out = plan->impl.scheme;
    return MNN_OK;
}

int mnn_conv_plan_candidates(mnn_conv_plan_t plan, mnn_scheme* out, int32_t cap, int32_t* count)
{
    if (!plan || !count || cap < 0 || (cap > 0 && !out)) return fail(MNN_E_INVALID_ARG, "bad argument");
    *count = (int32_t)plan->cands.size();
    for (int i = 0; i < cap && i < (int)plan->cands.size(); ++i) out[i] = plan->cands[i];
    return MNN_OK;
}

int mnn_conv_plan_describe(mnn_conv_plan_t plan, char* buf, size_t cap)
{
    if (!plan || !buf || cap == 0) return fail(MNN_E_INVALID_ARG, "bad argument");
    describe_impl(plan->impl, buf, cap);
    return MNN_OK;
}

int mnn_conv_plan_info(mnn_conv_plan_t plan, mnn_plan_info* out)
{
    if (!plan || !out) return fail(MNN_E_INVALID_ARG, "NULL argument");
    std::memset(out, 0, sizeof *out);
    const Impl& im = plan->impl;
    if (im.scheme.kind == MNN_SCHEME_WINOGRAD) {
        out->alpha = im.wg.alpha; out->tile_n = im.wg.n; out->tiles_h = im.wg.th; out->tiles_w = im.wg.tw;
        out->alpha_w = im.wg.alpha_w; out->tile_n_w = im.wg.nw;
        out->p = im.wg.P; out->ldp = im.wg.ldp; out->kg = im.wg.kg; out->pg = im.wg.pg;
    }
    out->ldk = im.ldk;
    out->h_out = plan->L.Ho; out->w_out = plan->L.Wo;
    return MNN_OK;
}

size_t mnn_conv_workspace_bytes(mnn_conv_plan_t plan) { return plan ? plan->impl.bytes() : 0; }

int mnn_conv_run(mnn_conv_plan_t plan, const float* input, const float* weight, const float* bias, float* output,
                 void* stream)
{
    int rc = check_run_args(plan, input, weight, output);
    if (rc) return rc;
    hipStream_t s = (hipStream_t)stream;
    Impl& im = plan->impl;
    if (!plan->weights_valid || plan->cached_weight != weight) {
        if ((rc = im.run_stage(MNN_STAGE_FILTER, input, weight, bias, output, s))) return rc;
        plan->cached_weight = weight;
        plan->weights_valid = true;
    }
    for (int st = MNN_STAGE_INPUT; st < MNN_STAGE_COUNT; ++st)
        if ((rc = im.run_stage(st, input, weight, bias, output, s))) return rc;
    return MNN_OK;
}

int mnn_conv_run_stage(mnn_conv_plan_t plan, int32_t stage, const float* input, const float* weight,
                       const float* bias, float* output, void* stream)
{
    int rc = check_run_args(plan, input, weight, output);
    if (rc) return rc;
    if (stage < 0 || stage >= MNN_STAGE_COUNT) return fail(MNN_E_INVALID_ARG, "unknown stage %d", stage);
    rc = plan->impl.run_stage(stage, input, weight, bias, output, (hipStream_t)stream);
    if (!rc && stage == MNN_STAGE_FILTER) { plan->cached_weight = weight; plan->weights_valid = true; }
    return rc;
}

int mnn_conv_run_timed(mnn_conv_plan_t plan, const float* input, const float* weight, const float* bias,
                       float* output, void* stream, int32_t iters, float* stage_ms)
{
    int rc = check_run_args(plan, input, weight, output);
    if (rc) return rc;
    if (iters <= 0 || !stage_ms) return fail(MNN_E_INVALID_ARG, "iters must be positive and stage_ms not NULL");
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t ev[MNN_STAGE_COUNT + 1] = {};
    hipError_t e = hipSuccess;
    for (auto& v : ev)
        if ((e = hipEventCreate(&v)) != hipSuccess) break;
    double acc[MNN_STAGE_COUNT] = {};
    if (e == hipSuccess) {
        for (int it = 0; it < iters && !rc; ++it) {
            for (int st = 0; st < MNN_STAGE_COUNT && !rc; ++st) {
                if ((e = hipEventRecord(ev[st], s)) != hipSuccess) break;
                rc = plan->impl.run_stage(st, input, weight, bias, output, s);
            }
            if (rc || e != hipSuccess) break;
            if ((e = hipEventRecord(ev[MNN_STAGE_COUNT], s)) != hipSuccess) break;
            if ((e = hipEventSynchronize(ev[MNN_STAGE_COUNT])) != hipSuccess) break;
            for (int st = 0; st < MNN_STAGE_COUNT; ++st) {
                float ms = 0.f;
                if ((e = hipEventElapsedTime(&ms, ev[st], ev[st + 1])) != hipSuccess) break;
                if (plan->impl.has_stage(st)) acc[st] += ms;
            }
            if (e != hipSuccess) break;
        }
    }
    for (auto& v : ev)
        if (v) (void)hipEventDestroy(v);
    if (rc) return rc;
    if (e != hipSuccess) return fail_hip(e, "event timing");
    plan->cached_weight = weight;
    plan->weights_valid = true;
    for (int st = 0; st < MNN_STAGE_COUNT; ++st) stage_ms[st] = (float)(acc[st] / iters);
    return MNN_OK;
}

int mnn_conv_invalidate_weights(mnn_conv_plan_t plan)
{
    if (!plan) return fail(MNN_E_INVALID_ARG, "plan is NULL");
    plan->weights_valid = false;
    plan->cached_weight = nullptr;
    return MNN_OK;
}

int mnn_conv_plan_buffer(mnn_conv_plan_t plan, int32_t which, void** ptr, size_t* bytes)
{
    if (!plan || !ptr || !bytes) return fail(MNN_E_INVALID_ARG, "NULL argument");
    const Impl& im = plan->impl;
    switch (which) {
        case MNN_BUF_U: *ptr = im.U; *bytes = im.U_bytes; break;
        case MNN_BUF_V: *ptr = im.V; *bytes = im.V_bytes; break;
        case MNN_BUF_M: *ptr = im.M; *bytes = im.M_bytes; break;
        default: return fail(MNN_E_INVALID_ARG, "unknown buffer %d", which);
    }
    return MNN_OK;
}

int mnn_conv_read_buffer(mnn_conv_plan_t plan, int32_t which, void* dst, size_t bytes, void* stream)
{
    void* src = nullptr;
    size_t have = 0;
    int rc = mnn_conv_plan_buffer(plan, which, &src, &have);
    if (rc) return rc;
    if (!dst) return fail(MNN_E_INVALID_ARG, "dst is NULL");
    if (!src || bytes > have) return fail(MNN_E_INVALID_ARG, "the plan has no such buffer or it is smaller than %zu bytes", bytes);
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "hipStreamSynchronize");
    if ((e = hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost)) != hipSuccess) return fail_hip(e, "hipMemcpy");
    return MNN_OK;
}

void mnn_conv_plan_destroy(mnn_conv_plan_t plan) { delete plan; }

int mnn_conv_get_transforms(int32_t n, int32_t k, float f, float* AT, float* G, float* BT)
{
    if (!AT || !G || !BT) return fail(MNN_E_INVALID_ARG, "NULL output");
    if (n < 1 || k < 1 || !(f > 0.f)) return fail(MNN_E_INVALID_ARG, "n, k and f must be positive");
    WinogradMatrices m;
    try {
        if (!generate_winograd(n, k, (double)f, &m))
            return fail(MNN_E_UNSUPPORTED, "F(%d,%d): alpha = %d is outside 2..%d", n, k, n + k - 1, kMaxAlpha);  // the generator itself goes further than the kernels
    } catch (...) {
        return fail(MNN_E_OOM, "host allocation failed");
    }
    std::memcpy(AT, m.AT.data(), m.AT.size() * sizeof(float));
    std::memcpy(G, m.G.data(), m.G.size() * sizeof(float));
    std::memcpy(BT, m.BT.data(), m.BT.size() * sizeof(float));
    return MNN_OK;
}

int mnn_conv_analytic_cost(int32_t k, int32_t i_c, int32_t o_c, int32_t o_h, int32_t o_w, int32_t n, double* cost)
{
    if (!cost || k < 1 || i_c < 1 || o_c < 1 || o_h < 1 || o_w < 1 || n < 1) return fail(MNN_E_INVALID_ARG, "bad argument");
    *cost = analytic_cost(k, i_c, o_c, o_h, o_w, n);
    return MNN_OK;
}

int mnn_conv_analytic_tile(int32_t k, int32_t i_c, int32_t o_c, int32_t o_h, int32_t o_w, int32_t alpha_max,
                           int32_t* n_hat)
{
    if (!n_hat || k < 1 || i_c < 1 || o_c < 1 || o_h < 1 || o_w < 1 || alpha_max < k)
        return fail(MNN_E_INVALID_ARG, "bad argument");
    *n_hat = analytic_tile(k, i_c, o_c, o_h, o_w, alpha_max);
    return MNN_OK;
}

int mnn_conv_enumerate(const mnn_conv_shape* shape, const mnn_conv_geom* geom, const mnn_conv_options* options,
                       mnn_scheme* out, int32_t cap, int32_t* count)
{
    if (!count || cap < 0 || (cap > 0 && !out)) return fail(MNN_E_INVALID_ARG, "bad argument");
    Layer L;
    int rc = validate(shape, geom, &L);
    if (rc) return rc;
    mnn_conv_options o;
    if ((rc = validate_options(options, &o))) return rc;
    try {
        std::vector<mnn_scheme> c = enumerate(L, o);
        *count = (int32_t)c.size();
        for (int i = 0; i < cap && i < (int)c.size(); ++i) out[i] = c[i];
    } catch (...) {
        return fail(MNN_E_OOM, "host allocation failed");
    }
    return MNN_OK;
}

int mnn_conv_select(const mnn_scheme* cands, int32_t count, int32_t k, int32_t* chosen)
{
    if (!cands || count <= 0 || !chosen) return fail(MNN_E_INVALID_ARG, "bad argument");
    const int pick = select_scheme(cands, count, k);
    if (pick < 0) return fail(MNN_E_INVALID_ARG, "no candidate carries a time");
    *chosen = pick;
    return MNN_OK;
}

int mnn_gemm_f32(const mnn_gemm_desc* d, const float* At, const float* B, const float* bias, float* D, void* stream)
{
    if (!d || !At || !B || !D) return fail(MNN_E_INVALID_ARG, "NULL argument");
    GemmProblem p{};
    p.At = At; p.B = B; p.D = D; p.bias = bias;
    p.M = d->M; p.Ncols = d->ncols; p.R = d->R; p.batch = d->batch; p.lda = d->lda; p.L = d->L;
    p.variant = d->variant;
    p.prec = d->prec;
    if (p.prec < MNN_GEMM_FP32 || p.prec > MNN_GEMM_BF16X3) return fail(MNN_E_INVALID_ARG, "unknown precision %d", p.prec);
    p.strideA_batch = d->strideA_batch;
    p.strideB_batch = d->strideB_batch; p.strideB_img = d->strideB_img; p.strideB_row = d->strideB_row;
    p.strideD_batch = d->strideD_batch; p.strideD_img = d->strideD_img; p.strideD_row = d->strideD_row;
    hipError_t e = launch_gemm_f32(p, (hipStream_t)stream);
    if (e == hipErrorInvalidValue) { (void)hipGetLastError(); return fail(MNN_E_INVALID_ARG, "GEMM descriptor rejected (sizes, lda, alignment or variant)"); }
    if (e != hipSuccess) return fail_hip(e, "gemm launch");
    return MNN_OK;
}

struct mnn_strassen_s { Strassen impl; };

int mnn_strassen_levels_by_rule(int32_t M, int32_t R, int32_t ncols, int32_t max_levels)
{
    if (M <= 0 || R <= 0 || ncols <= 0 || max_levels < 0) return 0;
    return strassen_levels(M, R, ncols, max_levels);
}

int mnn_strassen_create(const mnn_gemm_desc* d, int32_t levels, void* stream, mnn_strassen_t* out)
{
    if (!d || !out) return fail(MNN_E_INVALID_ARG, "NULL argument");
    *out = nullptr;
    if (d->M <= 0 || d->ncols <= 0 || d->R <= 0 || d->L <= 0 || d->lda < d->M) return fail(MNN_E_INVALID_ARG, "bad GEMM descriptor");
    if (d->prec != MNN_GEMM_FP32) return fail(MNN_E_UNSUPPORTED, "Strassen runs on the fp32 GEMM only");
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        return fail(MNN_E_NO_DEVICE, "no HIP device available");
    }
    GemmProblem p{};
    p.M = d->M; p.Ncols = d->ncols; p.R = d->R; p.batch = d->batch; p.lda = d->lda; p.L = d->L;
    p.variant = d->variant; p.prec = d->prec;
    p.strideA_batch = d->strideA_batch;
    p.strideB_batch = d->strideB_batch; p.strideB_img = d->strideB_img; p.strideB_row = d->strideB_row;
    p.strideD_batch = d->strideD_batch; p.strideD_img = d->strideD_img; p.strideD_row = d->strideD_row;
    mnn_strassen_s* h = new (std::nothrow) mnn_strassen_s();
    if (!h) return fail(MNN_E_OOM, "host allocation failed");
    int rc;
    try {
        rc = h->impl.init(p, levels, (hipStream_t)stream);
    } catch (const std::bad_alloc&) {
        rc = fail(MNN_E_OOM, "host allocation failed");
    }
    if (rc) { delete h; return rc; }
    *out = h;
    return MNN_OK;
}

int mnn_strassen_set_left(mnn_strassen_t h, const float* At, void* stream)
{
    if (!h) return fail(MNN_E_INVALID_ARG, "handle is NULL");
    if (At && (reinterpret_cast<uintptr_t>(At) & 15u)) return fail(MNN_E_INVALID_ARG, "At must be 16-byte aligned");
    return h->impl.set_left(At, (hipStream_t)stream);
}

int mnn_strassen_run(mnn_strassen_t h, const float* B, const float* bias, float* D, void* stream)
{
    if (!h) return fail(MNN_E_INVALID_ARG, "handle is NULL");
    return h->impl.run(B, bias, D, (hipStream_t)stream);
}

int mnn_strassen_info(mnn_strassen_t h, int32_t* levels, int32_t* launches, size_t* workspace_bytes)
{
    if (!h) return fail(MNN_E_INVALID_ARG, "handle is NULL");
    if (levels) *levels = h->impl.levels;
    if (launches) *launches = h->impl.launches();
    if (workspace_bytes) *workspace_bytes = h->impl.bytes;
    return MNN_OK;
}

void mnn_strassen_destroy(mnn_strassen_t h) { delete h; }

int mnn_gemm_variant_count(int32_t prec)
{
    return (prec < MNN_GEMM_FP32 || prec > MNN_GEMM_BF16X3) ? 0 : gemm_variant_count(prec);
}

const char* mnn_gemm_variant_name(int32_t prec, int32_t variant)
{
    return (prec < MNN_GEMM_FP32 || prec > MNN_GEMM_BF16X3) ? nullptr : gemm_variant_name(prec, variant);
}

int mnn_conv_get_device_model(mnn_device_model* out)
{
    if (!out) return fail(MNN_E_INVALID_ARG, "out is NULL");
    std::lock_guard<std::mutex> lk(g_model_mu);
    *out = g_model;
    return MNN_OK;
}

int mnn_conv_set_device_model(const mnn_device_model* m)
{
    if (!m || !(m->flops > 0.0) || !(m->bytes_per_s > 0.0) || !(m->t_schedule_ms >= 0.0))
        return fail(MNN_E_INVALID_ARG, "flops and bytes_per_s must be positive, t_schedule_ms not negative");
    std::lock_guard<std::mutex> lk(g_model_mu);
    g_model = *m;
    return MNN_OK;
}

int mnn_conv_calibrate(void* stream, mnn_device_model* out)
{
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        return fail(MNN_E_NO_DEVICE, "no HIP device available");
    }
    hipStream_t s = (hipStream_t)stream;
    const int M = 4096, R = 2048, N = 4096;
    const size_t copy_bytes = (size_t)256 << 20;
    float *a = nullptr, *b = nullptr, *d = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = MNN_OK;
    mnn_device_model m{};
    do {
        if ((e = hipMalloc((void**)&a, (size_t)R * M * 4)) != hipSuccess || (e = hipMalloc((void**)&b, copy_bytes)) != hipSuccess ||
            (e = hipMalloc((void**)&d, copy_bytes)) != hipSuccess || (e = hipMemset(a, 0, (size_t)R * M * 4)) != hipSuccess ||
            (e = hipMemset(b, 0, copy_bytes)) != hipSuccess || (e = hipEventCreate(&e0)) != hipSuccess ||
            (e = hipEventCreate(&e1)) != hipSuccess) {
            rc = fail_hip(e, "calibration set-up");
            break;
        }
        auto timed = [&](int reps, const std::function<hipError_t()>& launch, double* ms_each) -> int {
            hipError_t er = launch();                                    // warm-up
            if (er == hipSuccess) er = hipEventRecord(e0, s);
            for (int i = 0; i < reps && er == hipSuccess; ++i) er = launch();
            if (er == hipSuccess) er = hipEventRecord(e1, s);
            if (er == hipSuccess) er = hipEventSynchronize(e1);
            float ms = 0.f;
            if (er == hipSuccess) er = hipEventElapsedTime(&ms, e0, e1);
            if (er != hipSuccess) return fail_hip(er, "calibration run");
            *ms_each = (double)ms / reps;
            return MNN_OK;
        };
        GemmProblem p{};
        p.At = a; p.B = b; p.D = d; p.M = M; p.Ncols = N; p.R = R; p.batch = 1; p.lda = M; p.L = N;
        p.strideB_row = N; p.strideD_row = N;
        GemmChoice c{0, 1};
        if ((rc = tune_gemm(p, s, &c))) break;
        p.variant = c.variant;                                           // 4096 tiles: never split
        double ms = 0.0;
        if ((rc = timed(5, [&] { return launch_gemm_f32(p, s); }, &ms))) break;
        m.flops = 2.0 * M * R * N / (ms * 1e-3);
        if ((rc = timed(5, [&] { return hipMemcpyAsync(d, b, copy_bytes, hipMemcpyDeviceToDevice, s); }, &ms))) break;
        m.bytes_per_s = 2.0 * (double)copy_bytes / (ms * 1e-3);
        if ((rc = timed(200, [&] { return launch_weight_transpose(a, d, 1, 1, 4, s); }, &ms))) break;
        m.t_schedule_ms = ms;
    } while (false);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (a) (void)hipFree(a);
    if (b) (void)hipFree(b);
    if (d) (void)hipFree(d);
    if (rc) return rc;
    if ((rc = mnn_conv_set_device_model(&m))) return rc;
    if (out) *out = m;
    return MNN_OK;
}

int mnn_conv_predict_ms(const mnn_conv_shape* shape, const mnn_conv_geom* geom, const mnn_scheme* scheme, double* ms)
{
    if (!scheme || !ms) return fail(MNN_E_INVALID_ARG, "NULL argument");
    Layer L;
    int rc = validate(shape, geom, &L);
    if (rc) return rc;
    if (scheme->kind == MNN_SCHEME_WINOGRAD && (!winograd_admissible(L) || scheme->tile_n < 2))
        return fail(MNN_E_UNSUPPORTED, "not a Winograd layer or tile");
    if (scheme->kind == MNN_SCHEME_GEMM1X1 && !is_pointwise(L)) return fail(MNN_E_UNSUPPORTED, "not a 1x1 layer");
    if (scheme->kind < MNN_SCHEME_DIRECT || scheme->kind > MNN_SCHEME_GEMM1X1) return fail(MNN_E_INVALID_ARG, "unknown scheme kind");
    *ms = predict_ms(L, *scheme);
    return MNN_OK;
}

int mnn_conv_cache_size(void)
{
    std::lock_guard<std::mutex> lk(g_cache_mu);
    return (int)g_cache.size();
}

void mnn_conv_cache_clear(void)
{
    std::lock_guard<std::mutex> lk(g_cache_mu);
    g_cache.clear();
}

int mnn_conv_cache_save(const char* path)
{
    if (!path) return fail(MNN_E_INVALID_ARG, "path is NULL");
    FILE* f = std::fopen(path, "w");
    if (!f) return fail(MNN_E_INVALID_ARG, "cannot open %s for writing", path);
    std::fprintf(f, "mnnconv-plan-cache 2\n");
    {
        std::lock_guard<std::mutex> lk(g_cache_mu);
        for (const auto& kv : g_cache) {
            const std::vector<int>& v = std::get<1>(kv.first);
            std::fprintf(f, "S %d %zu", std::get<0>(kv.first), v.size());
            for (int x : v) std::fprintf(f, " %d", x);
            std::fprintf(f, " %.9g | %d %d %d %d %.6g\n", (double)std::get<2>(kv.first), kv.second.kind, kv.second.tile_n,
                         kv.second.prec, kv.second.variant, (double)kv.second.est_ms);
        }
    }
    {
        std::lock_guard<std::mutex> lk(g_gemm_mu);
        for (const auto& kv : g_gemm_choice) {
            const std::vector<long long>& v = std::get<1>(kv.first);
            std::fprintf(f, "G %d %zu", std::get<0>(kv.first), v.size());
            for (long long x : v) std::fprintf(f, " %lld", x);
            std::fprintf(f, " | %d %d\n", kv.second.variant, kv.second.splitk);
        }
    }
    const bool ok = std::fclose(f) == 0;
    return ok ? MNN_OK : fail(MNN_E_INVALID_ARG, "error writing %s", path);
}

int mnn_conv_cache_load(const char* path)
{
    if (!path) return fail(MNN_E_INVALID_ARG, "path is NULL");
    FILE* f = std::fopen(path, "r");
    if (!f) return fail(MNN_E_INVALID_ARG, "cannot open %s", path);
    int version = 0;
    int rc = MNN_OK;
    try {
        if (std::fscanf(f, "mnnconv-plan-cache %d", &version) != 1 || version != 2) {
            rc = fail(MNN_E_INVALID_ARG, "%s is not a plan cache of this library", path);
        } else {
            char tag[4];
            while (!rc && std::fscanf(f, "%3s", tag) == 1) {
                int dev = 0;
                size_t n = 0;
                if (std::fscanf(f, "%d %zu", &dev, &n) != 2 || n > 64) { rc = fail(MNN_E_INVALID_ARG, "malformed entry in %s", path); break; }
                if (tag[0] == 'S') {
                    std::vector<int> v(n);
                    for (size_t i = 0; i < n && !rc; ++i)
                        if (std::fscanf(f, "%d", &v[i]) != 1) rc = fail(MNN_E_INVALID_ARG, "malformed entry in %s", path);
                    double fscale = 0, est = 0;
                    mnn_scheme sc{};
                    if (!rc && std::fscanf(f, "%lf | %d %d %d %d %lf", &fscale, &sc.kind, &sc.tile_n, &sc.prec, &sc.variant, &est) != 6)
                        rc = fail(MNN_E_INVALID_ARG, "malformed entry in %s", path);
                    if (!rc) {
                        sc.est_ms = (float)est;
                        std::lock_guard<std::mutex> lk(g_cache_mu);
                        g_cache[CacheKey(dev, v, (float)fscale)] = sc;
                    }
                } else if (tag[0] == 'G') {
                    std::vector<long long> v(n);
                    for (size_t i = 0; i < n && !rc; ++i)
                        if (std::fscanf(f, "%lld", &v[i]) != 1) rc = fail(MNN_E_INVALID_ARG, "malformed entry in %s", path);
                    int variant = 0, splitk = 1;
                    if (!rc && std::fscanf(f, " | %d %d", &variant, &splitk) != 2) rc = fail(MNN_E_INVALID_ARG, "malformed entry in %s", path);
                    if (!rc && (splitk < 1 || splitk > 64)) rc = fail(MNN_E_INVALID_ARG, "bad split in %s", path);
                    const int vprec = v.empty() ? 0 : (int)v.back();
                    if (!rc && (vprec < 0 || vprec > MNN_GEMM_BF16X3 || variant < 0 || variant >= gemm_variant_count(vprec)))
                        rc = fail(MNN_E_INVALID_ARG, "unknown GEMM configuration %d in %s", variant, path);
                    if (!rc) {
                        std::lock_guard<std::mutex> lk(g_gemm_mu);
                        g_gemm_choice[GemmKey(dev, v)] = GemmChoice{variant, splitk};
                    }
                } else {
                    rc = fail(MNN_E_INVALID_ARG, "unknown entry type in %s", path);
                }
            }
        }
    } catch (...) {
        rc = fail(MNN_E_OOM, "host allocation failed");
    }
    std::fclose(f);
    return rc;
}

const char* mnn_last_error(void) { return g_err.c_str(); }

int mnn_version(void) { return 100; }

}  // extern "C"

// ------------------------------------------------------------------ chain of layers
namespace {

int chain_create_impl(const mnn_chain_layer* layers, int32_t n_layers, const mnn_conv_options* options, void* stream,
                      mnn_chain_t* out_chain)
{
    if (!out_chain) return fail(MNN_E_INVALID_ARG, "out_chain must not be NULL");
    *out_chain = nullptr;
    if (!layers || n_layers <= 0 || n_layers > 4096) return fail(MNN_E_INVALID_ARG, "layers must not be NULL, 1 <= n_layers <= 4096");
    mnn_conv_options o;
    int rc = validate_options(options, &o);
    if (rc) return rc;
    std::unique_ptr<mnn_chain_s> ch(new mnn_chain_s());
    ch->opt = o;
    for (int i = 0; i < n_layers; ++i) {
        Layer L;
        if ((rc = validate(&layers[i].shape, &layers[i].geom, &L))) return rc;
        if (i > 0) {
            const Layer& p = ch->layers.back();
            if (L.s.n != p.s.n || L.s.c_in != p.s.c_out || L.s.h != p.Ho || L.s.w != p.Wo)
                return fail(MNN_E_INVALID_ARG, "layer %d takes [%d,%d,%d,%d] but layer %d produces [%d,%d,%d,%d]", i, L.s.n,
                            L.s.c_in, L.s.h, L.s.w, i - 1, p.s.n, p.s.c_out, p.Ho, p.Wo);
        }
        ch->layers.push_back(L);
    }
    // pre-inference per layer: an ordinary plan times the candidates (or finds them cached) and leaves
    // the scheme and the GEMM configuration in the caches; its own workspace is released again
    std::vector<mnn_scheme> chosen(n_layers);
    for (int i = 0; i < n_layers; ++i) {
        mnn_conv_plan_t pl = nullptr;
        if ((rc = plan_impl(&layers[i].shape, &layers[i].geom, &o, stream, &pl))) return rc;
        chosen[i] = pl->impl.scheme;
        delete pl;
    }
    hipError_t e = hipGetDevice(&ch->device);
    if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
    const int n = n_layers;
    ch->bias.assign(n, nullptr);
    ch->has_bias.assign(n, 0);
    ch->weights_set.assign(n, 0);
    for (int i = 0; i < n; ++i) {
        ch->impls.emplace_back(new Impl());
        Impl& im = *ch->impls.back();
        if ((rc = im.prepare(ch->layers[i], chosen[i], o, /*external_transient=*/true))) return rc;
        if ((rc = im.tune((hipStream_t)stream))) return rc;
        const size_t bb = (size_t)ch->layers[i].s.c_out * sizeof(float);
        if ((e = hipMalloc((void**)&ch->bias[i], bb)) != hipSuccess) return fail_hip(e, "hipMalloc bias");
        ch->weight_bytes += im.U_bytes + bb;
    }
    // the virtual walk: activation i lives over layers i and i+1, workspace i over layer i
    std::vector<ArenaBuffer> bufs;
    ch->act_bytes.assign(n, 0);
    for (int i = 0; i + 1 < n; ++i) {
        const Layer& L = ch->layers[i];
        ch->act_bytes[i] = (size_t)L.s.n * L.s.c_out * L.Ho * L.Wo * sizeof(float);
        bufs.push_back(ArenaBuffer{(long long)ch->act_bytes[i], i, i + 1});
    }
    for (int i = 0; i < n; ++i) bufs.push_back(ArenaBuffer{(long long)ch->impls[i]->transient_bytes(), i, i});
    std::vector<long long> off;
    long long total = 0;
    if (!plan_arena(bufs, 256, &off, &total)) return fail(MNN_E_INVALID_ARG, "arena planning failed");
    ch->act_off.assign(off.begin(), off.begin() + (n - 1));
    ch->ws_off.assign(off.begin() + (n - 1), off.end());
    ch->arena_bytes = (size_t)total;
    std::vector<long long> live(n, 0);
    for (const ArenaBuffer& b : bufs) {
        const long long sz = (b.bytes + 255) / 256 * 256;
        ch->unshared_bytes += (size_t)sz;
        for (int t = b.first; t <= b.last; ++t) live[t] += sz;
    }
    ch->live_peak_bytes = (size_t)*std::max_element(live.begin(), live.end());
    if (total > 0) {
        if ((e = hipMalloc((void**)&ch->arena, (size_t)total)) != hipSuccess) return fail_hip(e, "hipMalloc arena");
        if ((e = hipMemset(ch->arena, 0, (size_t)total)) != hipSuccess) return fail_hip(e, "hipMemset arena");
        if ((e = hipDeviceSynchronize()) != hipSuccess) return fail_hip(e, "hipDeviceSynchronize");
    }
    for (int i = 0; i < n; ++i) ch->impls[i]->bind_transient(ch->arena + ch->ws_off[i]);
    *out_chain = ch.release();
    return MNN_OK;
}

int chain_check(mnn_chain_t ch, int32_t layer)
{
    if (!ch) return fail(MNN_E_INVALID_ARG, "chain is NULL");
    if (layer < 0 || layer >= (int)ch->impls.size()) return fail(MNN_E_INVALID_ARG, "layer %d out of range", layer);
    return MNN_OK;
}

int chain_ready(mnn_chain_t ch)
{
    if (!ch) return fail(MNN_E_INVALID_ARG, "chain is NULL");
    for (size_t i = 0; i < ch->weights_set.size(); ++i)
        if (!ch->weights_set[i]) return fail(MNN_E_INVALID_ARG, "weights of layer %d have not been set", (int)i);
    return MNN_OK;
}

}  // namespace

extern "C" {

int mnn_chain_create(const mnn_chain_layer* layers, int32_t n_layers, const mnn_conv_options* options, void* stream,
                     mnn_chain_t* out_chain)
{
    try {
        return chain_create_impl(layers, n_layers, options, stream, out_chain);
    } catch (const std::bad_alloc&) {
        return fail(MNN_E_OOM, "host allocation failed");
    } catch (...) {
        return fail(MNN_E_INVALID_ARG, "unexpected exception in mnn_chain_create");
    }
}

int mnn_chain_set_weights(mnn_chain_t ch, int32_t layer, const float* weight, const float* bias, void* stream)
{
    int rc = chain_check(ch, layer);
    if (rc) return rc;
    if (!weight) return fail(MNN_E_INVALID_ARG, "weight must not be NULL");
    hipStream_t s = (hipStream_t)stream;
    if ((rc = ch->impls[layer]->run_stage(MNN_STAGE_FILTER, nullptr, weight, nullptr, nullptr, s))) return rc;
    if (bias) {
        hipError_t e = hipMemcpyAsync(ch->bias[layer], bias, (size_t)ch->layers[layer].s.c_out * sizeof(float),
                                      hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return fail_hip(e, "hipMemcpyAsync bias");
    }
    ch->has_bias[layer] = bias ? 1 : 0;
    ch->weights_set[layer] = 1;
    return MNN_OK;
}

int mnn_chain_run(mnn_chain_t ch, const float* input, float* output, void* stream)
{
    int rc = chain_ready(ch);
    if (rc) return rc;
    if (!input || !output) return fail(MNN_E_INVALID_ARG, "input and output must not be NULL");
    return ch->enqueue(input, output, (hipStream_t)stream);
}

int mnn_chain_capture(mnn_chain_t ch, const float* input, float* output)
{
    int rc = chain_ready(ch);
    if (rc) return rc;
    if (!input || !output) return fail(MNN_E_INVALID_ARG, "input and output must not be NULL");
    hipError_t e;
    if (!ch->capture_stream &&
        (e = hipStreamCreateWithFlags(&ch->capture_stream, hipStreamNonBlocking)) != hipSuccess)
        return fail_hip(e, "hipStreamCreateWithFlags");
    if (ch->exec) { (void)hipGraphExecDestroy(ch->exec); ch->exec = nullptr; }
    if (ch->graph) { (void)hipGraphDestroy(ch->graph); ch->graph = nullptr; }
    ch->graph_nodes = 0;
    if ((e = hipStreamBeginCapture(ch->capture_stream, hipStreamCaptureModeThreadLocal)) != hipSuccess)
        return fail_hip(e, "hipStreamBeginCapture");
    rc = ch->enqueue(input, output, ch->capture_stream);
    hipGraph_t g = nullptr;
    e = hipStreamEndCapture(ch->capture_stream, &g);
    if (rc) {
        if (g) (void)hipGraphDestroy(g);
        return rc;
    }
    if (e != hipSuccess || !g) return fail_hip(e, "hipStreamEndCapture");
    ch->graph = g;
    if ((e = hipGraphInstantiate(&ch->exec, g, nullptr, nullptr, 0)) != hipSuccess) {
        ch->exec = nullptr;
        return fail_hip(e, "hipGraphInstantiate");
    }
    size_t nodes = 0;
    if (hipGraphGetNodes(g, nullptr, &nodes) == hipSuccess) ch->graph_nodes = nodes;
    return MNN_OK;
}

int mnn_chain_replay(mnn_chain_t ch, void* stream)
{
    if (!ch) return fail(MNN_E_INVALID_ARG, "chain is NULL");
    if (!ch->exec) return fail(MNN_E_INVALID_ARG, "mnn_chain_capture has not been called");
    hipError_t e = hipGraphLaunch(ch->exec, (hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "hipGraphLaunch");
    return MNN_OK;
}

int mnn_chain_info(mnn_chain_t ch, mnn_chain_info_t* out)
{
    if (!ch || !out) return fail(MNN_E_INVALID_ARG, "NULL argument");
    std::memset(out, 0, sizeof *out);
    out->n_layers = (int32_t)ch->impls.size();
    out->kernels_per_run = ch->kernels_per_run();
    out->graph_nodes = (int32_t)ch->graph_nodes;
    out->arena_bytes = ch->arena_bytes;
    out->unshared_bytes = ch->unshared_bytes;
    out->live_peak_bytes = ch->live_peak_bytes;
    out->weight_bytes = ch->weight_bytes;
    return MNN_OK;
}

int mnn_chain_layer_scheme(mnn_chain_t ch, int32_t layer, mnn_scheme* out)
{
    int rc = chain_check(ch, layer);
    if (rc) return rc;
    if (!out) return fail(MNN_E_INVALID_ARG, "out is NULL");
    *out = ch->impls[layer]->scheme;
    return MNN_OK;
}

int mnn_chain_layer_describe(mnn_chain_t ch, int32_t layer, char* buf, size_t cap)
{
    int rc = chain_check(ch, layer);
    if (rc) return rc;
    if (!buf || cap == 0) return fail(MNN_E_INVALID_ARG, "bad argument");
    describe_impl(*ch->impls[layer], buf, cap);
    return MNN_OK;
}

int mnn_chain_read_activation(mnn_chain_t ch, int32_t layer, float* dst, size_t bytes, void* stream)
{
    int rc = chain_check(ch, layer);
    if (rc) return rc;
    if (layer + 1 >= (int)ch->impls.size()) return fail(MNN_E_INVALID_ARG, "the last layer writes to the caller's output");
    if (!dst || bytes > ch->act_bytes[layer]) return fail(MNN_E_INVALID_ARG, "dst NULL or more bytes than the activation holds");
    hipError_t e = hipStreamSynchronize((hipStream_t)stream);
    if (e != hipSuccess) return fail_hip(e, "hipStreamSynchronize");
    if ((e = hipMemcpy(dst, ch->arena + ch->act_off[layer], bytes, hipMemcpyDeviceToHost)) != hipSuccess)
        return fail_hip(e, "hipMemcpy");
    return MNN_OK;
}

void mnn_chain_destroy(mnn_chain_t ch) { delete ch; }

int mnn_arena_plan(const int64_t* bytes, const int32_t* first, const int32_t* last, int32_t count, int64_t align,
                   int64_t* offsets, int64_t* total)
{
    if (count < 0 || !total || (count > 0 && (!bytes || !first || !last || !offsets)))
        return fail(MNN_E_INVALID_ARG, "NULL argument or negative count");
    try {
        std::vector<ArenaBuffer> bufs(count);
        for (int i = 0; i < count; ++i) bufs[i] = ArenaBuffer{(long long)bytes[i], first[i], last[i]};
        std::vector<long long> off;
        long long tot = 0;
        if (!plan_arena(bufs, (long long)align, &off, &tot))
            return fail(MNN_E_INVALID_ARG, "need bytes >= 0, 0 <= first <= last and align a power of two");
        for (int i = 0; i < count; ++i) offsets[i] = off[i];
        *total = tot;
        return MNN_OK;
    } catch (const std::bad_alloc&) {
        return fail(MNN_E_OOM, "host allocation failed");
    }
}

}  // extern "C"
