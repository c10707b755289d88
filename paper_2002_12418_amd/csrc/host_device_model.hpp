// The operator cost of Section 3.2 (2) with measured device constants.
// Private part of api.cpp (included there once, in order); everything lives in its unnamed namespace.
#pragma once

namespace {

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
        const double n = s.tile_n;
        const double nh = wino_axis_n(L.s.kh, s.tile_n), nw = wino_axis_n(L.s.kw, s.tile_n);
        const double ah = nh + L.s.kh - 1, aw = nw + L.s.kw - 1;
        (void)n;
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

}  // namespace
