// Tile configuration (and split of the reduction) of the GEMM stage, chosen by timing per matrix shape.
// Private part of api.cpp (included there once, in order); everything lives in its unnamed namespace.
#pragma once

namespace {

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
    std::vector<std::pair<float, GemmChoice>> timed;                     // every configuration that ran
    int rc = MNN_OK;
    const bool tune_log = std::getenv("MNNCONV_TUNE_LOG") != nullptr;    // one line per timed configuration on stderr
    for (int v = 1; v < gemm_variant_count(p.prec) && !rc; ++v) {
        p.variant = v;
        p.splitk = 1; p.splitk_partial = nullptr;
        float ms = -1.f;
        if ((rc = time_gemm(p, s, e0, e1, iters, &ms))) break;
        if (ms >= 0.f && (best_ms < 0.f || ms < best_ms)) { best_ms = ms; best = GemmChoice{v, 1}; }
        if (ms >= 0.f) timed.emplace_back(ms, GemmChoice{v, 1});
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
            if (!rc && ms >= 0.f) timed.emplace_back(ms, GemmChoice{v, sk});
            if (tune_log && !rc && ms >= 0.f)
                std::fprintf(stderr, "[mnnconv tune]     %s splitk=%d: %.2f us\n", gemm_variant_name(p.prec, v), sk, ms * 1e3f / iters);
        }
    }
    // One pass of 4 launches separates configurations that differ by 10 %, not those that differ by 2 %
    // (clock and cache state drift over the pass).  The configurations within 8 % of the fastest (at most four)
    // are timed again in five interleaved rounds; the least time of each decides.
    if (!rc && best_ms > 0.f) {
        std::sort(timed.begin(), timed.end(), [](const auto& a, const auto& b) { return a.first < b.first; });
        size_t nf = 0;
        while (nf < timed.size() && nf < 4 && timed[nf].first <= 1.08f * best_ms) ++nf;
        if (nf > 1) {
            int max_sk = 1;
            for (size_t i = 0; i < nf; ++i) max_sk = std::max(max_sk, timed[i].second.splitk);
            float* part = nullptr;
            if (max_sk > 1) {
                long long pf = 0;
                for (size_t i = 0; i < nf; ++i) {
                    p.variant = timed[i].second.variant;
                    pf = std::max(pf, gemm_splitk_workspace(p, timed[i].second.splitk));
                }
                if ((e = hipMalloc((void**)&part, (size_t)pf * sizeof(float))) != hipSuccess) rc = fail_hip(e, "hipMalloc split-K scratch");
            }
            for (int round = 0; round < 5 && !rc; ++round)
                for (size_t i = 0; i < nf && !rc; ++i) {
                    p.variant = timed[i].second.variant;
                    p.splitk = timed[i].second.splitk;
                    p.splitk_partial = p.splitk > 1 ? part : nullptr;
                    float ms = -1.f;
                    rc = time_gemm(p, s, e0, e1, iters, &ms);
                    if (!rc && ms >= 0.f && (round == 0 || ms < timed[i].first)) timed[i].first = ms;
                }
            if (part) (void)hipFree(part);
            if (!rc) {
                size_t bi = 0;
                for (size_t i = 1; i < nf; ++i)
                    if (timed[i].first < timed[bi].first) bi = i;
                best = timed[bi].second;
                if (tune_log)
                    std::fprintf(stderr, "[mnnconv tune]   finalists %zu -> %s splitk=%d: %.2f us\n", nf,
                                 gemm_variant_name(p.prec, best.variant), best.splitk, timed[bi].first * 1e3f / iters);
            }
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

}  // namespace
