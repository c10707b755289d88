// Host side of Strassen's algorithm (Section 3.3.2): operand buffers per level, launch order.
// Private part of api.cpp (included there once, in order); everything lives in its unnamed namespace.
#pragma once

namespace {

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
                (e = hipMalloc((void**)&td, db)) != hipSuccess ||
                (e = launch_fill_pattern(ta, ab / sizeof(float), 0x59u, -0.5f, 0.5f, s)) != hipSuccess ||
                (e = launch_fill_pattern(tb, bb / sizeof(float), 0x5au, -1.f, 1.f, s)) != hipSuccess)
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
            const size_t nb = (size_t)pow7(levels);
            if ((e = launch_fill_pattern(Ax[levels], nb * Rl(levels) * Ml(levels), 0x5du, -0.5f, 0.5f, s)) != hipSuccess ||
                (e = launch_fill_pattern(Bx[levels], nb * Rl(levels) * Nl(levels), 0x5eu, -1.f, 1.f, s)) != hipSuccess)
                return fail_hip(e, "Strassen tuning operand fill");
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

}  // namespace
