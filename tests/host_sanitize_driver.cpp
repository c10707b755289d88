// Host-only exercise of the C ABI, built with AddressSanitizer and UndefinedBehaviorSanitizer by
// tests/test_host_sanitizers.py: generator, enumeration, selection, cost model, arena planner, cache files and
// the error paths, on seeded pseudo-random arguments (valid and invalid).  Needs no GPU.
#include "mnn_conv.h"
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <vector>
int main()
{
    int checks = 0;
    // generator for every admissible (n, k)
    for (int k = 1; k <= 7; ++k)
        for (int n = 1; n + k - 1 <= 10; ++n)
            for (float f : {0.5f, 1.0f, 0.425f, 0.0f}) {
                int a = n + k - 1;
                std::vector<float> AT(n * a), G(a * k), BT(a * a);
                int rc = mnn_conv_get_transforms(n, k, f, AT.data(), G.data(), BT.data());
                if (rc != 0 && f != 0.0f) { std::printf("transforms(%d,%d,%g) -> %d %s\n", n, k, f, rc, mnn_last_error()); }
                ++checks;
            }
    mnn_conv_get_transforms(0, 3, 0.5f, nullptr, nullptr, nullptr);
    mnn_conv_get_transforms(9, 3, 0.5f, nullptr, nullptr, nullptr);
    // enumeration over many shapes and options
    std::mt19937 rng(7);
    for (int it = 0; it < 3000; ++it) {
        mnn_conv_shape s{(int)(rng() % 33), (int)(rng() % 600), (int)(rng() % 130), (int)(rng() % 130), (int)(rng() % 600),
                         (int)(rng() % 9), (int)(rng() % 9)};
        mnn_conv_geom g{(int)(rng() % 3), (int)(rng() % 3), (int)(rng() % 4), (int)(rng() % 4), (int)(rng() % 3), (int)(rng() % 3)};
        mnn_conv_options o;
        mnn_conv_options_default(&o);
        o.alpha_max = 4 + rng() % 8;
        o.allow_bf16 = rng() % 2;
        o.point_scale_f = (rng() % 2) ? 0.f : 0.5f;
        mnn_scheme c[256];
        int32_t cnt = 0;
        int rc = mnn_conv_enumerate(&s, &g, (rng() % 4) ? &o : nullptr, c, 256, &cnt);
        if (rc == 0) {
            int32_t chosen = -1;
            for (int i = 0; i < cnt; ++i) c[i].est_ms = (float)(rng() % 1000) / 100.f - 1.f;
            mnn_conv_select(c, cnt, s.kh > s.kw ? s.kh : s.kw, &chosen);
            for (int i = 0; i < cnt; ++i) { double ms = 0; mnn_conv_predict_ms(&s, &g, &c[i], &ms); }
            mnn_conv_plan_t p = nullptr;
            rc = mnn_conv_plan(&s, &g, &o, nullptr, &p);      // no device: must fail cleanly
            if (rc == 0) mnn_conv_plan_destroy(p);
        }
        // small cap
        mnn_conv_enumerate(&s, &g, &o, c, (int)(rng() % 3), &cnt);
        ++checks;
    }
    // analytic cost
    for (int it = 0; it < 2000; ++it) {
        double cost = 0; int32_t nh = 0;
        mnn_conv_analytic_cost(rng() % 9, rng() % 600, rng() % 600, rng() % 200, rng() % 200, rng() % 12, &cost);
        mnn_conv_analytic_tile(rng() % 9, rng() % 600, rng() % 600, rng() % 200, rng() % 200, rng() % 12, &nh);
        mnn_strassen_levels_by_rule(rng() % 5000, rng() % 5000, rng() % 5000, rng() % 6);
        ++checks;
    }
    // arena planner
    for (int it = 0; it < 500; ++it) {
        int n = rng() % 40;
        std::vector<int64_t> bytes(n), off(n);
        std::vector<int32_t> first(n), last(n);
        for (int i = 0; i < n; ++i) { bytes[i] = rng() % 100000; first[i] = rng() % 20; last[i] = first[i] + rng() % 5; }
        int64_t total = 0;
        int rc = mnn_arena_plan(bytes.data(), first.data(), last.data(), n, 256, off.data(), &total);
        if (rc == 0)
            for (int i = 0; i < n; ++i)
                for (int j = i + 1; j < n; ++j)
                    if (bytes[i] && bytes[j] && first[i] <= last[j] && first[j] <= last[i] && off[i] < off[j] + bytes[j] && off[j] < off[i] + bytes[i]) {
                        std::printf("arena overlap!\n"); return 1;
                    }
        ++checks;
    }
    // cache file round trip with garbage
    const char* path = "mnn_san_cache.txt";   // in the working directory the test gives us
    mnn_conv_cache_save(path);
    mnn_conv_cache_load(path);
    FILE* f = std::fopen(path, "w");
    std::fprintf(f, "mnnconv-plan-cache 3\nS 0 999999999 1 2 3\nG 0 3 1 2\nS 0 16 1 2 3 4 5 6 7 8 9 10 11 12 13 14 15 16 0.5 | 2 4 0 0 0.1\n\x01\x02garbage");
    std::fclose(f);
    int rc = mnn_conv_cache_load(path);
    std::printf("garbage cache load -> %d (%s)\n", rc, mnn_last_error());
    mnn_conv_cache_load("/nonexistent/file");
    mnn_conv_cache_save(nullptr);
    mnn_conv_cache_clear();
    // misc
    mnn_device_model m;
    mnn_conv_get_device_model(&m);
    m.flops = -1;
    mnn_conv_set_device_model(&m);
    mnn_conv_set_device_model(nullptr);
    mnn_measure_device_peaks(nullptr, nullptr);
    for (int prec = -1; prec < 4; ++prec)
        for (int v = -1; v < mnn_gemm_variant_count(prec) + 1; ++v) mnn_gemm_variant_name(prec, v);
    // the calls that prepare weights or run without a plan: no device here, every path must fail cleanly
    mnn_conv_set_weights(nullptr, nullptr, nullptr);
    {
        float dummy[4] = {};
        mnn_conv_shape sh{1, 4, 9, 9, 4, 3, 3};
        mnn_conv_geom ge{1, 1, 1, 1, 1, 1};
        for (int tile = -1; tile <= 9; ++tile) mnn_conv_run_static(&sh, &ge, tile, dummy, dummy, nullptr, dummy, nullptr);
        mnn_conv_shape big{16, 256, 128, 128, 256, 3, 3};
        int rcs = mnn_conv_run_static(&big, &ge, 4, dummy, dummy, nullptr, dummy, nullptr);
        if (rcs != MNN_E_UNSUPPORTED) { std::printf("static entry point accepted a layer beyond its scratch array (%d)\n", rcs); return 1; }
        mnn_conv_run_static(nullptr, nullptr, 2, nullptr, nullptr, nullptr, nullptr, nullptr);
        if (mnn_conv_static_scratch_bytes() != ((size_t)64 << 20)) return 1;
    }
    mnn_chain_t ch = nullptr;
    mnn_chain_create(nullptr, 0, nullptr, nullptr, &ch);
    mnn_chain_layer cl[2] = {};
    mnn_chain_create(cl, 2, nullptr, nullptr, &ch);
    mnn_chain_destroy(nullptr);
    mnn_conv_plan_destroy(nullptr);
    mnn_strassen_destroy(nullptr);
    std::printf("done, %d checks, version %d\n", checks, mnn_version());
    return 0;
}
