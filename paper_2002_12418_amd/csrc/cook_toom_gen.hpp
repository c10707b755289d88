// Host-side Winograd generator: transform matrices A^T, G, B^T of F(n, k) for any
// output tile n and kernel size k (Section 3.3.1 item (3) of the MNN paper).
//
// Interpolation points are the roots of x (x-f)(x+f)(x-2f)(x+2f)..., i.e.
// p_m = i_m * f with integer indices i = 0, +1, -1, +2, -2, ...; the first
// alpha - 1 = n + k - 2 of them are used together with the point at infinity.
//
// Because every point is an integer multiple of f, each matrix entry factors
// into (ratio of integers) * f^e:
//     A^T[i][j] = i_j^i * f^i
//     G[j][l]   = i_j^l / D_j * f^(l - (alpha-2)),   D_j = prod_{m != j} (i_j - i_m)
//     B^T[j][t] = (-1)^(alpha-2-t) e_{alpha-2-t}(i without i_j) * f^(alpha-2-t)
// (e_r = elementary symmetric polynomial), and the infinity row / column are
//     A^T[n-1][alpha-1] = 1,  G[alpha-1][k-1] = 1,
//     B^T[alpha-1][t]   = (-1)^(alpha-1-t) e_{alpha-1-t}(all i) * f^(alpha-1-t).
// The integer parts are evaluated exactly in 64-bit integers; the result is
// rounded once to double and once to float.
#pragma once
#include <cmath>
#include <cstdint>
#include <vector>

namespace mnnconv {

constexpr int kMaxAlpha = 12;

struct WinogradMatrices {
    int n = 0, k = 0, alpha = 0;
    std::vector<float> AT;   // n x alpha
    std::vector<float> G;    // alpha x k
    std::vector<float> BT;   // alpha x alpha
};

inline std::vector<int64_t> point_indices(int count) {
    std::vector<int64_t> idx;
    idx.push_back(0);
    for (int64_t m = 1; (int)idx.size() < count; ++m) {
        idx.push_back(m);
        if ((int)idx.size() < count) idx.push_back(-m);
    }
    idx.resize(count);
    return idx;
}

// coefficients (ascending powers) of prod_r (x - roots[r]) over the integers
inline std::vector<int64_t> int_poly_from_roots(const std::vector<int64_t>& roots) {
    std::vector<int64_t> poly{1};
    for (int64_t r : roots) {
        std::vector<int64_t> next(poly.size() + 1, 0);
        for (size_t t = 0; t < poly.size(); ++t) {
            next[t + 1] += poly[t];
            next[t] -= r * poly[t];
        }
        poly.swap(next);
    }
    return poly;
}

inline int64_t ipow(int64_t b, int e) {
    int64_t r = 1;
    for (int i = 0; i < e; ++i) r *= b;
    return r;
}

// Returns false when (n, k) is outside the supported range.
inline bool generate_winograd(int n, int k, double f, WinogradMatrices* out) {
    if (n < 1 || k < 1 || !(f > 0.0) || !std::isfinite(f)) return false;
    const int alpha = n + k - 1;
    if (alpha < 2 || alpha > kMaxAlpha) return false;
    const int fin = alpha - 1;
    const std::vector<int64_t> idx = point_indices(fin);

    out->n = n; out->k = k; out->alpha = alpha;
    out->AT.assign((size_t)n * alpha, 0.f);
    out->G.assign((size_t)alpha * k, 0.f);
    out->BT.assign((size_t)alpha * alpha, 0.f);

    for (int j = 0; j < fin; ++j) {
        std::vector<int64_t> others;
        int64_t D = 1;
        for (int m = 0; m < fin; ++m) {
            if (m == j) continue;
            others.push_back(idx[m]);
            D *= (idx[j] - idx[m]);
        }
        const std::vector<int64_t> Mj = int_poly_from_roots(others);   // degree alpha-2, integer-index domain
        for (int i = 0; i < n; ++i)
            out->AT[(size_t)i * alpha + j] = (float)((double)ipow(idx[j], i) * std::pow(f, i));
        for (int l = 0; l < k; ++l)
            out->G[(size_t)j * k + l] =
                (float)(((double)ipow(idx[j], l) / (double)D) * std::pow(f, l - (alpha - 2)));
        // coefficient of x^t of prod (x - i_m f) is  Mj[t] * f^(deg - t)
        for (int t = 0; t <= alpha - 2; ++t)
            out->BT[(size_t)j * alpha + t] = (float)((double)Mj[t] * std::pow(f, (alpha - 2) - t));
    }
    const std::vector<int64_t> Mall = int_poly_from_roots(idx);        // degree alpha-1
    out->AT[(size_t)(n - 1) * alpha + (alpha - 1)] = 1.f;
    out->G[(size_t)(alpha - 1) * k + (k - 1)] = 1.f;
    for (int t = 0; t <= alpha - 1; ++t)
        out->BT[(size_t)(alpha - 1) * alpha + t] = (float)((double)Mall[t] * std::pow(f, (alpha - 1) - t));
    return true;
}

}  // namespace mnnconv
