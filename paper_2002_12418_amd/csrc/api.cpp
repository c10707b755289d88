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

#include "host_core.hpp"
#include "host_device_model.hpp"
#include "host_gemm_tune.hpp"
#include "host_strassen.hpp"
#include "host_conv_impl.hpp"

namespace {

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
                         : (st == MNN_STAGE_GEMM && im->gemm_splitk > 1) ? 2                    // + the slice reduction
                         : (st == MNN_STAGE_GEMM && im->scheme.kind == MNN_SCHEME_WINOGRAD && im->scheme.variant != MNN_WINO_UNFUSED)
                               ? wino_fused_launch_count(im->wg, im->scheme.variant - 1) : 1;
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
                // scratch tensors for the timing launches
                Scratch sc;
                const size_t xb = (size_t)L.s.n * L.s.c_in * L.s.h * L.s.w * sizeof(float);
                const size_t wb = (size_t)L.s.c_out * L.s.c_in * L.s.kh * L.s.kw * sizeof(float);
                const size_t yb = (size_t)L.s.n * L.s.c_out * L.Ho * L.Wo * sizeof(float);
                if ((e = hipMalloc((void**)&sc.x, xb)) != hipSuccess || (e = hipMalloc((void**)&sc.w, wb)) != hipSuccess ||
                    (e = hipMalloc((void**)&sc.y, yb)) != hipSuccess) {
                    delete plan;
                    return fail_hip(e, "hipMalloc planner scratch");
                }
                // seeded values with the spread of real activations and He-initialised weights: the time of the
                // matrix-core stage depends on the operand bits (power, sustained clock), all-zero tensors flatter it
                const float wr = std::sqrt(6.f / (float)(L.s.c_in * L.s.kh * L.s.kw));
                if ((e = launch_fill_pattern(sc.x, xb / sizeof(float), 0x2002u, -1.f, 1.f, s)) != hipSuccess ||
                    (e = launch_fill_pattern(sc.w, wb / sizeof(float), 0x12418u, -wr, wr, s)) != hipSuccess) {
                    delete plan;
                    return fail_hip(e, "planner scratch fill");
                }
                double best_pred = -1.0;
                int last_skip = MNN_E_OOM;
                for (const auto& c : plan->cands) {
                    const double pm = predict_ms(L, c);
                    if (best_pred < 0.0 || pm < best_pred) best_pred = pm;
                }
                for (auto& c : plan->cands) {
                    if (o.prune_ratio > 1.f && predict_ms(L, c) > (double)o.prune_ratio * best_pred) { c.est_ms = -1.f; continue; }
                    rc = time_candidate(L, o, &c, sc, s);
                    // a scheme that does not fit in memory or that the kernels do not cover for this shape is not a
                    // candidate; the cheapest of those that apply is selected (Section 3.2 (1))
                    if (rc == MNN_E_OOM || rc == MNN_E_UNSUPPORTED) { c.est_ms = -1.f; (void)hipGetLastError(); last_skip = rc; continue; }
                    if (rc) { delete plan; return rc; }
                }
                const int pick = select_scheme(plan->cands.data(), (int)plan->cands.size(), wino_k(L));
                if (pick < 0) {
                    delete plan;
                    return fail(last_skip == MNN_E_UNSUPPORTED ? MNN_E_UNSUPPORTED : MNN_E_OOM, "no candidate scheme could be timed");
                }
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
        out->tiled = im.wg.tiled; out->pb = im.wg.pb;
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

size_t mnn_conv_static_scratch_bytes(void) { return kStaticScratchBytes; }

int mnn_conv_run_static(const mnn_conv_shape* shape, const mnn_conv_geom* geom, int32_t tile_n, const float* input,
                        const float* weight, const float* bias, float* output, void* stream)
{
    if (!input || !weight || !output) return fail(MNN_E_INVALID_ARG, "input, weight and output must not be NULL");
    Layer L;
    int rc = validate(shape, geom, &L);
    if (rc) return rc;
    if (tile_n < 0) return fail(MNN_E_INVALID_ARG, "tile_n must be 0 (no Winograd) or the n of F(n,k)");
    mnn_conv_options o;
    default_options(&o);
    o.alpha_max = kMaxAlphaT;
    const mnn_scheme sc = tile_n > 0 ? make_scheme(MNN_SCHEME_WINOGRAD, tile_n, MNN_GEMM_FP32, MNN_WINO_UNFUSED)
                                     : make_scheme(is_pointwise(L) ? MNN_SCHEME_GEMM1X1 : MNN_SCHEME_DIRECT, 0, MNN_GEMM_FP32);
    try {
        Impl im;                                   // host object only: every device buffer is bound below
        if ((rc = im.prepare(L, sc, o, /*external_transient=*/true, /*external_persistent=*/true))) return rc;
        const size_t need = im.external_bytes();
        if (need > kStaticScratchBytes)
            return fail(MNN_E_UNSUPPORTED, "this layer needs %zu bytes of scratch memory, the static buffer holds %zu: plan it with "
                        "mnn_conv_plan instead", need, (size_t)kStaticScratchBytes);
        float* base = nullptr;
        hipError_t e = static_scratch(&base);
        if (e != hipSuccess) return fail_hip(e, "static scratch buffer");
        im.bind_external(reinterpret_cast<char*>(base));
        hipStream_t s = (hipStream_t)stream;
        // the buffer keeps the last call's contents: the padding of the prepared weights and of V must read as zero
        // (by a kernel, not a memset: the call may be recorded into a graph)
        if ((e = launch_fill_zero(base, (Impl::align256(im.U_bytes) + Impl::align256(im.V_bytes)) / sizeof(float), s)) != hipSuccess)
            return fail_hip(e, "scratch clear");
        for (int st = MNN_STAGE_FILTER; st < MNN_STAGE_COUNT; ++st)
            if ((rc = im.run_stage(st, input, weight, bias, output, s))) return rc;
        return MNN_OK;
    } catch (const std::bad_alloc&) {
        return fail(MNN_E_OOM, "host allocation failed");
    }
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

int mnn_conv_set_weights(mnn_conv_plan_t plan, const float* weight, void* stream)
{
    if (!plan) return fail(MNN_E_INVALID_ARG, "plan is NULL");
    if (!weight) return fail(MNN_E_INVALID_ARG, "weight must not be NULL");
    int rc = plan->impl.run_stage(MNN_STAGE_FILTER, nullptr, weight, nullptr, nullptr, (hipStream_t)stream);
    if (rc) return rc;
    plan->cached_weight = weight;
    plan->weights_valid = true;
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
            (e = hipMalloc((void**)&d, copy_bytes)) != hipSuccess ||
            (e = launch_fill_pattern(a, (size_t)R * M, 0x5bu, -0.5f, 0.5f, s)) != hipSuccess ||
            (e = launch_fill_pattern(b, copy_bytes / sizeof(float), 0x5cu, -1.f, 1.f, s)) != hipSuccess || (e = hipEventCreate(&e0)) != hipSuccess ||
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

int mnn_measure_device_peaks(void* stream, mnn_device_peaks* out)
{
    if (!out) return fail(MNN_E_INVALID_ARG, "out is NULL");
    int ndev = 0;
    hipError_t e = hipGetDeviceCount(&ndev);
    if (e != hipSuccess || ndev <= 0) {
        (void)hipGetLastError();
        return fail(MNN_E_NO_DEVICE, "no HIP device available");
    }
    hipStream_t s = (hipStream_t)stream;
    hipDeviceProp_t prop{};
    int dev = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess || (e = hipGetDeviceProperties(&prop, dev)) != hipSuccess)
        return fail_hip(e, "device properties");
    const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const int wgs = cus * 8, iters = 2048;                               // 8 waves per SIMD, 4*iters instructions per wave
    const size_t copy_bytes = (size_t)256 << 20;
    float *b = nullptr, *d = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = MNN_OK;
    mnn_device_peaks m{};
    do {
        if ((e = hipMalloc((void**)&b, copy_bytes)) != hipSuccess || (e = hipMalloc((void**)&d, copy_bytes)) != hipSuccess) {
            (void)hipGetLastError();
            rc = fail(MNN_E_OOM, "device peaks: %s", hipGetErrorString(e));
            break;
        }
        if ((e = hipMemsetAsync(b, 0, copy_bytes, s)) != hipSuccess || (e = hipEventCreate(&e0)) != hipSuccess ||
            (e = hipEventCreate(&e1)) != hipSuccess) {
            rc = fail_hip(e, "device peaks set-up");
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
            if (er != hipSuccess) return fail_hip(er, "device peaks run");
            *ms_each = (double)ms / reps;
            return MNN_OK;
        };
        double ms = 0.0;
        if ((rc = timed(3, [&] { return launch_mfma_issue(d, wgs, iters, s); }, &ms))) break;
        m.mfma_f32_flops = (double)wgs * 4 * (4.0 * iters) * (2.0 * 32 * 32 * 2) / (ms * 1e-3);
        if ((rc = timed(10, [&] { return launch_stream_copy(b, d, copy_bytes / 4, s); }, &ms))) break;
        m.copy_bytes_per_s = 2.0 * (double)copy_bytes / (ms * 1e-3);
    } while (false);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (b) (void)hipFree(b);
    if (d) (void)hipFree(d);
    if (rc) return rc;
    *out = m;
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
    std::fprintf(f, "mnnconv-plan-cache 3\n");
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
    {
        std::lock_guard<std::mutex> lk(g_input_cap_mu);
        for (const auto& kv : g_input_cap) {
            const std::vector<int>& v = std::get<1>(kv.first);
            std::fprintf(f, "I %d %zu", std::get<0>(kv.first), v.size());
            for (int x : v) std::fprintf(f, " %d", x);
            std::fprintf(f, " | %d\n", kv.second);
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
        if (std::fscanf(f, "mnnconv-plan-cache %d", &version) != 1 || version != 3) {
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
                } else if (tag[0] == 'I') {
                    std::vector<int> v(n);
                    for (size_t i = 0; i < n && !rc; ++i)
                        if (std::fscanf(f, "%d", &v[i]) != 1) rc = fail(MNN_E_INVALID_ARG, "malformed entry in %s", path);
                    int cap = 0;
                    if (!rc && std::fscanf(f, " | %d", &cap) != 1) rc = fail(MNN_E_INVALID_ARG, "malformed entry in %s", path);
                    if (!rc && !(cap == 0 || (cap >= 8 && cap <= 32))) rc = fail(MNN_E_INVALID_ARG, "bad wavefront cap in %s", path);
                    if (!rc) {
                        std::lock_guard<std::mutex> lk(g_input_cap_mu);
                        g_input_cap[InputCapKey(dev, v)] = cap;
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

int mnn_version(void) { return 110; }

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
