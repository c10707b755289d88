// One realised scheme for one layer: its buffers, its GEMM problem, its stages.
// Private part of api.cpp (included there once, in order); everything lives in its unnamed namespace.
#pragma once

namespace {

// Input-transform occupancy cap per (device, geometry), chosen by timing like the GEMM tile configuration.
using InputCapKey = std::tuple<int, std::vector<int>>;
std::mutex g_input_cap_mu;
std::map<InputCapKey, int> g_input_cap;

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
    // The prepared weights live as long as the plan and are the plan's own allocation, except for the single-shot
    // entry point that may not allocate: there U, too, is bound to a region of the caller-independent scratch array.
    bool persistent_external = false;

    ~Impl() { release(); }
    Impl() = default;
    Impl(const Impl&) = delete;
    Impl& operator=(const Impl&) = delete;

    void release()
    {
        if (U && !persistent_external) (void)hipFree(U);
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

    int alloc_persistent(float** p, size_t bytes, const char* what)
    {
        if (persistent_external) { *p = nullptr; return MNN_OK; }
        return alloc_zero(p, bytes, what);
    }

    static size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }
    // everything bound from outside (persistent_external): U first, then the transient buffers
    size_t external_bytes() const { return align256(U_bytes) + transient_bytes(); }
    void bind_external(char* base)
    {
        U = reinterpret_cast<float*>(base);
        bind_transient(base + align256(U_bytes));
    }

    size_t transient_bytes() const { return align256(V_bytes) + align256(M_bytes) + align256(sk_partial_bytes); }
    void bind_transient(char* base)
    {
        V = V_bytes ? reinterpret_cast<float*>(base) : nullptr;
        M = M_bytes ? reinterpret_cast<float*>(base + align256(V_bytes)) : nullptr;
        sk_partial = sk_partial_bytes ? reinterpret_cast<float*>(base + align256(V_bytes) + align256(M_bytes)) : nullptr;
    }

    int prepare(const Layer& layer, const mnn_scheme& s, const mnn_conv_options& o, bool external_transient = false,
                bool external_persistent = false)
    {
        L = layer;
        scheme = s;
        transient_external = external_transient;
        persistent_external = external_persistent;
        const mnn_conv_shape& sh = L.s;
        ldk = round_up(sh.c_out, 4);
        if (s.prec != MNN_GEMM_FP32 && s.kind == MNN_SCHEME_WINOGRAD && s.variant != MNN_WINO_UNFUSED)
            return fail(MNN_E_UNSUPPORTED, "the fused Winograd kernels multiply in fp32 only");
        if (s.kind == MNN_SCHEME_WINOGRAD) {
            if (!winograd_admissible(L))
                return fail(MNN_E_UNSUPPORTED, "Winograd needs a kernel with more than one tap, stride 1, dilation 1");
            rect = winograd_rect(L);
            const int n = s.tile_n, k = wino_k(L);
            if (!wino_tile_available(L, n))
                return fail(MNN_E_UNSUPPORTED, "F(%d,.) is outside the built range for a %d x %d kernel (n 2..8, k 2..7, alpha <= %d; "
                            "alpha <= 8 with several taps on both axes)", n, sh.kh, sh.kw, kMaxAlphaT);
            // one matrix set per axis; an axis with a single tap keeps the 1 x 1 identity.
            // f = 0: the scale with the least fp32 error for this alpha.  Up to alpha = 8 that is the paper's 0.5;
            // for 9 and 10 points spaced 0.425 apart bring the error down 3-5x (points further out blow up G, points
            // closer together blow up B^T).
            auto axis_matrices = [&](int k_axis, WinogradMatrices* out) -> bool {
                if (k_axis == 1) {
                    out->n = out->k = out->alpha = 1;
                    out->AT.assign(1, 1.f); out->G.assign(1, 1.f); out->BT.assign(1, 1.f);
                    return true;
                }
                const double f = o.point_scale_f > 0.f ? (double)o.point_scale_f : (n + k_axis - 1 >= 9 ? 0.425 : 0.5);
                return generate_winograd(n, k_axis, f, out);
            };
            if (!axis_matrices(sh.kh, &mats) || !axis_matrices(sh.kw, &mats_w))
                return fail(MNN_E_UNSUPPORTED, "generator rejected F(%d,%d)", n, k);
            wg.N = sh.n; wg.C = sh.c_in; wg.H = sh.h; wg.W = sh.w; wg.K = sh.c_out;
            wg.Ho = L.Ho; wg.Wo = L.Wo; wg.pad_h = L.g.pad_h; wg.pad_w = L.g.pad_w;
            wg.n = mats.n; wg.k = mats.k; wg.alpha = mats.alpha;
            wg.nw = mats_w.n; wg.kw = mats_w.k; wg.alpha_w = mats_w.alpha;
            wg.th = (L.Ho + wg.n - 1) / wg.n; wg.tw = (L.Wo + wg.nw - 1) / wg.nw;
            const long long P = (long long)sh.n * wg.th * wg.tw;
            if (P >= (1ll << 30)) return fail(MNN_E_UNSUPPORTED, "too many tiles");
            wg.P = (int)P; wg.ldp = round_up(wg.P, 4); wg.ldk = ldk;
            // Tiled row layout for V and M ([channel][64 tiles][position][tile in block]): what one wavefront of a transform
            // kernel writes or reads is then one contiguous 16 KB run instead of alpha^2 runs of 256 bytes (input transform
            // 3-7 % faster, output transform up to 10 % on the large layers).  Not for few tiles (a block pads P to 64), and
            // only while one position's operand, which now spans all of V, stays within the GEMM loader's 2 GiB window.
            if (!rect && s.variant == MNN_WINO_UNFUSED && wg.P >= 1024) {
                const long long pb = (wg.P + 63) / 64;
                const long long v_bytes = (long long)wg.alpha * wg.alpha_w * sh.c_in * pb * 64 * (long long)sizeof(float);
                if (v_bytes < (1ll << 31) - 4096) { wg.tiled = 1; wg.pb = (int)pb; wg.ldp = (int)pb * 64; }
            }
            const size_t a2 = (size_t)wg.alpha * wg.alpha_w;
            if (rect && s.variant != MNN_WINO_UNFUSED)
                return fail(MNN_E_UNSUPPORTED, "kernels that are not square have no fused variant");
            if (!rect && !wino_variant_available(n, k, s.variant))
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
                if ((rc = alloc_persistent(&U, U_bytes, "hipMalloc U"))) return rc;
                if ((rc = alloc_transient(&V, V_bytes, "hipMalloc V"))) return rc;
                // asks the runtime once how many 64 x 64 workgroups the device holds, here and not in the first launch
                // (which may be recorded into a graph)
                (void)wino_fused_launch_count(wg, s.variant - 1);
                return MNN_OK;
            }
            if ((long long)wg.C * wg.ldp >= (1ll << 31) || (long long)wg.K * wg.ldp >= (1ll << 31))
                return fail(MNN_E_UNSUPPORTED, "Winograd-domain plane too large");
            U_bytes = a2 * sh.c_in * ldk * sizeof(float);
            V_bytes = a2 * sh.c_in * wg.ldp * sizeof(float);
            M_bytes = a2 * sh.c_out * wg.ldp * sizeof(float);
            if ((rc = alloc_persistent(&U, U_bytes, "hipMalloc U"))) return rc;
            if ((rc = alloc_transient(&V, V_bytes, "hipMalloc V"))) return rc;
            if ((rc = alloc_transient(&M, M_bytes, "hipMalloc M"))) return rc;
            return MNN_OK;
        }
        if (s.kind == MNN_SCHEME_GEMM1X1) {
            if (!is_pointwise(L)) return fail(MNN_E_UNSUPPORTED, "GEMM scheme needs a 1x1 kernel, stride 1, no padding");
            if ((long long)sh.n * sh.h * sh.w >= (1ll << 31)) return fail(MNN_E_UNSUPPORTED, "too many pixels");
            U_bytes = (size_t)sh.c_in * ldk * sizeof(float);
            return alloc_persistent(&U, U_bytes, "hipMalloc Wt");
        }
        if (s.kind == MNN_SCHEME_DIRECT) {
            // implicit GEMM on the matrix cores: weights transposed to [C*kh*kw][ldk]
            if ((long long)sh.n * L.Ho * L.Wo >= (1ll << 31) || (long long)sh.n * sh.c_in * sh.h * sh.w >= (1ll << 31))
                return fail(MNN_E_UNSUPPORTED, "tensor too large for the sliding-window kernel");
            U_bytes = (size_t)sh.c_in * sh.kh * sh.kw * ldk * sizeof(float);
            int rcd = alloc_persistent(&U, U_bytes, "hipMalloc Wt");
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
        if (wg.tiled) {
            // V[c][p/64][xi][p%64]: position xi starts 64 floats in, a run of 64 columns is contiguous, the next run
            // lies alpha^2 * 64 floats on, the next channel pb runs on
            const long long a2 = (long long)wg.alpha * wg.alpha_w;
            p.L = 64;
            p.strideB_batch = 64; p.strideB_img = a2 * 64; p.strideB_row = (long long)wg.pb * a2 * 64;
            p.strideD_batch = 64; p.strideD_img = a2 * 64; p.strideD_row = (long long)wg.pb * a2 * 64;
        }
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

    // Resident wavefronts per CU of the input transform (WinoGeom::itx_waves), remembered per geometry.  What is timed is the
    // transform inside whole per-inference passes on scratch tensors (input transform, multiplication, output transform), because
    // its time depends on what the kernels around it leave in the caches: a cap that wins when the kernel runs alone can lose in
    // sequence.  (The time of the whole pass is no usable criterion where the multiplication dominates: its run-to-run spread
    // exceeds what the cap moves.)
    int tune_input_cap(hipStream_t s)
    {
        if (scheme.kind != MNN_SCHEME_WINOGRAD || rect) return MNN_OK;
        int dev = 0;
        (void)hipGetDevice(&dev);
        const InputCapKey key(dev, std::vector<int>{wg.N, wg.C, wg.H, wg.W, wg.K, wg.n, wg.k, wg.pad_h, wg.pad_w, wg.blocked, wg.tiled,
                                                    scheme.variant, scheme.prec});
        {
            std::lock_guard<std::mutex> lk(g_input_cap_mu);
            auto it = g_input_cap.find(key);
            if (it != g_input_cap.end()) { wg.itx_waves = it->second; return MNN_OK; }
        }
        int cus = 256;
        (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        const long long lanes = wg.blocked ? (long long)wg.cchunks * ((wg.P + 15) / 16) * 64 : (long long)wg.C * wg.P;
        auto remember = [&](int cap) {
            wg.itx_waves = cap;
            std::lock_guard<std::mutex> lk(g_input_cap_mu);
            g_input_cap[key] = cap;
        };
        if (lanes / 256 < 8ll * cus) { remember(0); return MNN_OK; }          // a short grid never fills a CU that far
        if (transient_external || !V) { wg.itx_waves = 16; return MNN_OK; }      // nothing to time on: the usual optimum
        const size_t xb = (size_t)wg.N * wg.C * wg.H * wg.W * sizeof(float);
        const size_t yb = (size_t)wg.N * wg.K * wg.Ho * wg.Wo * sizeof(float);
        float *tx = nullptr, *ty = nullptr;
        constexpr int kMaxIters = 24;
        hipEvent_t ev[2 * kMaxIters] = {};
        hipError_t e = hipSuccess;
        int rc = MNN_OK, best = 0;
        float best_ms = -1.f;
        do {
            if ((e = hipMalloc((void**)&tx, xb)) != hipSuccess || (e = hipMalloc((void**)&ty, yb)) != hipSuccess) {
                rc = fail_hip(e, "hipMalloc tuning scratch");
                break;
            }
            if ((e = launch_fill_pattern(tx, xb / sizeof(float), 0x5fu, -1.f, 1.f, s)) != hipSuccess ||
                (e = launch_fill_pattern(U, U_bytes / sizeof(float), 0x60u, -0.5f, 0.5f, s)) != hipSuccess) {
                rc = fail_hip(e, "input transform tuning set-up");
                break;
            }
            for (auto& v : ev)
                if ((e = hipEventCreate(&v)) != hipSuccess) break;
            if (e != hipSuccess) { rc = fail_hip(e, "hipEventCreate"); break; }
            // one measurement: `iters` whole passes back to back (input transform, multiplication, output transform), the
            // input transform of each bracketed by events; returns the mean time of that stage in its natural surroundings
            auto measure = [&](int iters, float* stage_ms) -> int {
                for (int i = 0; i < iters; ++i) {
                    if ((e = hipEventRecord(ev[2 * i], s)) != hipSuccess) return fail_hip(e, "hipEventRecord");
                    int r = run_stage(MNN_STAGE_INPUT, tx, nullptr, nullptr, ty, s);
                    if (r) return r;
                    if ((e = hipEventRecord(ev[2 * i + 1], s)) != hipSuccess) return fail_hip(e, "hipEventRecord");
                    for (int st = MNN_STAGE_GEMM; st < MNN_STAGE_COUNT; ++st)
                        if ((r = run_stage(st, tx, nullptr, nullptr, ty, s))) return r;
                }
                if ((e = hipStreamSynchronize(s)) != hipSuccess) return fail_hip(e, "hipStreamSynchronize");
                double sum = 0.0;
                for (int i = 1; i < iters; ++i) {                                           // the first pass is the warm-up
                    float ms = 0.f;
                    if ((e = hipEventElapsedTime(&ms, ev[2 * i], ev[2 * i + 1])) != hipSuccess) return fail_hip(e, "hipEventElapsedTime");
                    sum += ms;
                }
                *stage_ms = (float)(sum / (iters - 1));
                return MNN_OK;
            };
            static const int caps[] = {0, 20, 16, 12, 10};
            const int ncaps = wg.blocked ? 4 : 5;
            float least[5] = {-1.f, -1.f, -1.f, -1.f, -1.f};
            // enough passes per measurement for about 1 ms of the stage: short layers are decided by differences of a microsecond
            float probe = 0.f;
            wg.itx_waves = 0;
            if ((rc = measure(4, &probe))) break;
            int iters = probe > 0.f ? (int)(1.0f / probe) + 1 : kMaxIters;
            iters = iters < 6 ? 6 : iters > kMaxIters ? kMaxIters : iters;
            for (int round = 0; round < 3 && !rc; ++round)
                for (int ci = 0; ci < ncaps && !rc; ++ci) {
                    wg.itx_waves = caps[ci];
                    float ms = 0.f;
                    if ((rc = measure(iters, &ms))) break;
                    if (least[ci] < 0.f || ms < least[ci]) least[ci] = ms;
                }
            // the least stage time decides; a cap has to win by 1 % to displace a weaker one
            for (int ci = 0; ci < ncaps && !rc; ++ci)
                if (best_ms < 0.f || least[ci] < best_ms * 0.99f) { best_ms = least[ci]; best = caps[ci]; }
            // the prepared weights go back to the zeros they held (their padding must read as zero)
            if (!rc && ((e = hipMemsetAsync(U, 0, U_bytes, s)) != hipSuccess || (e = hipStreamSynchronize(s)) != hipSuccess))
                rc = fail_hip(e, "tuning operand reset");
        } while (false);
        for (auto& v : ev)
            if (v) (void)hipEventDestroy(v);
        if (tx) (void)hipFree(tx);
        if (ty) (void)hipFree(ty);
        wg.itx_waves = 0;
        if (rc) return rc;
        remember(best);
        return MNN_OK;
    }

    int tune(hipStream_t s)
    {
        int rc = tune_gemm_stage(s);
        return rc ? rc : tune_input_cap(s);
    }

    int tune_gemm_stage(hipStream_t s)
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
            if (cached_gemm_choice(p, &c)) return adopt(p, c);
            // the tile configurations are timed on operands with the spread of real U and V, not on the zeros the
            // buffers hold after allocation (matrix-core power, and with it the clock, depends on the operand bits);
            // afterwards the buffers, padding included, are zero again
            hipError_t e;
            if ((e = launch_fill_pattern(U, U_bytes / sizeof(float), 0x55u, -0.5f, 0.5f, s)) != hipSuccess ||
                (e = launch_fill_pattern(V, V_bytes / sizeof(float), 0x56u, -2.f, 2.f, s)) != hipSuccess)
                return fail_hip(e, "tuning operand fill");
            int rc = tune_gemm(p, s, &c);
            if ((e = hipMemsetAsync(U, 0, U_bytes, s)) != hipSuccess || (e = hipMemsetAsync(V, 0, V_bytes, s)) != hipSuccess ||
                (e = hipStreamSynchronize(s)) != hipSuccess)
                return fail_hip(e, "tuning operand reset");
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
            if (!rc && ((e = launch_fill_pattern(tx, xb / sizeof(float), 0x57u, -1.f, 1.f, s)) != hipSuccess ||
                        (e = launch_fill_pattern(tb, (size_t)sh.c_out, 0x58u, -0.1f, 0.1f, s)) != hipSuccess))
                rc = fail_hip(e, "tuning scratch fill");
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
        if (e == hipErrorInvalidValue) {
            // a launcher's own check of what its kernel assumes (sizes, alignment, grid limits) said no
            (void)hipGetLastError();
            return fail(MNN_E_UNSUPPORTED, "stage %d of this scheme does not cover the layer's shape", st);
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
    char capbuf[32] = "";
    if (im.scheme.kind == MNN_SCHEME_WINOGRAD && im.wg.itx_waves > 0) std::snprintf(capbuf, sizeof capbuf, " input-waves/cu=%d", im.wg.itx_waves);
    const std::string tail = std::string(im.wg.tiled ? " tiled" : "") + capbuf;
    switch (im.scheme.kind) {
        case MNN_SCHEME_WINOGRAD:
            if (im.rect)
                std::snprintf(buf, cap, "F(%dx%d,%dx%d) unfused gemm=%s", im.wg.n, im.wg.nw, im.wg.k, im.wg.kw, gv);
            else if (im.scheme.variant == MNN_WINO_UNFUSED)
                std::snprintf(buf, cap, "F(%d,%d) unfused gemm=%s%s", im.wg.n, im.wg.k, gv, tail.c_str());
            else
                std::snprintf(buf, cap, "F(%d,%d) fused-output %s%s", im.wg.n, im.wg.k,
                              im.scheme.variant == MNN_WINO_FUSED_OUT_32 ? "32x32" : "64x64", tail.c_str());
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

}  // namespace
