// Winograd transforms for kernels that are not square, the rectangular case of Section 3.3.1 of the MNN paper
// ("kernels of any size"): every axis has its own generated matrix set,
//   U = G_h w G_w^T,   V = B_h^T d B_w,   Y = A_h^T [ sum_c U (.) V ] A_w,
// with alpha_h x alpha_w Winograd-domain positions.  Along an axis with a single tap (1 x k, k x 1 kernels) the
// matrices are the 1 x 1 identity and the transform is one-dimensional; with several taps on both axes
// (k_h x k_w, k_h != k_w) the output tile is n x n and alpha_h = n + k_h - 1, alpha_w = n + k_w - 1.
//
// Same mapping as the square kernels: one lane per (channel, tile), consecutive lanes are consecutive tiles,
// so stores of V and loads of M are contiguous across the wavefront.
#include <hip/hip_runtime.h>
#include "kernels.hpp"

namespace mnnconv {
namespace {

constexpr int kMaxK = 7;
constexpr int kMaxMixedAlpha = 8;      // k_h x k_w kernels with several taps on both axes are built up to alpha = 8

struct RectFilterMat { float gh[kMaxAlphaT][kMaxK], gw[kMaxAlphaT][kMaxK]; };

__global__ __launch_bounds__(256) void filter_transform_rect_kernel(WinoGeom g, RectFilterMat gm,
                                                                    const float* __restrict__ w, float* __restrict__ U)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)g.K * g.C) return;
    const int kk = (int)(idx % g.K);
    const int c = (int)(idx / g.K);
    const float* wp = w + ((long long)kk * g.C + c) * g.k * g.kw;
    for (int i = 0; i < g.alpha; ++i)
        for (int j = 0; j < g.alpha_w; ++j) {
            float acc = 0.f;
            for (int r = 0; r < g.k; ++r) {
                float row = 0.f;
                for (int s = 0; s < g.kw; ++s) row = fmaf(wp[r * g.kw + s], gm.gw[j][s], row);
                acc = fmaf(gm.gh[i][r], row, acc);
            }
            U[((long long)(i * g.alpha_w + j) * g.C + c) * g.ldk + kk] = acc;
        }
}

template <int AH, int AW>
__global__ __launch_bounds__(256) void input_transform_rect_kernel(WinoGeom g, MatArg<AH, AH> bh, MatArg<AW, AW> bw,
                                                                   const float* __restrict__ x, float* __restrict__ V)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)g.C * g.P) return;
    const int c = (int)(idx / g.P);
    const int p = (int)(idx % g.P);
    const int tx = p % g.tw;
    const int t2 = p / g.tw;
    const int ty = t2 % g.th;
    const int img = t2 / g.th;
    const int y0 = ty * g.n - g.pad_h;
    const int x0 = tx * g.nw - g.pad_w;
    const float* xp = x + ((long long)img * g.C + c) * g.H * g.W;
    float d[AH][AW];
#pragma unroll
    for (int i = 0; i < AH; ++i) {
        const int iy = y0 + i;
        const bool rowok = (iy >= 0) && (iy < g.H);
#pragma unroll
        for (int j = 0; j < AW; ++j) {
            const int ix = x0 + j;
            d[i][j] = (rowok && ix >= 0 && ix < g.W) ? xp[(long long)iy * g.W + ix] : 0.f;
        }
    }
    float t[AH][AW];                     // t = B_h^T d
#pragma unroll
    for (int i = 0; i < AH; ++i)
#pragma unroll
        for (int j = 0; j < AW; ++j) {
            float acc = 0.f;
#pragma unroll
            for (int a = 0; a < AH; ++a) acc = fmaf(bh.v[i][a], d[a][j], acc);
            t[i][j] = acc;
        }
    const long long plane = (long long)g.C * g.ldp;
    float* vp = V + (long long)c * g.ldp + p;
#pragma unroll
    for (int i = 0; i < AH; ++i)
#pragma unroll
        for (int j = 0; j < AW; ++j) {   // v = t B_w,  v[i][j] = sum_b t[i][b] B_w^T[j][b]
            float acc = 0.f;
#pragma unroll
            for (int b = 0; b < AW; ++b) acc = fmaf(t[i][b], bw.v[j][b], acc);
            vp[(long long)(i * AW + j) * plane] = acc;
        }
}

template <int NH, int NW, int AH, int AW>
__global__ __launch_bounds__(256) void output_transform_rect_kernel(WinoGeom g, MatArg<NH, AH> ah, MatArg<NW, AW> aw,
                                                                    const float* __restrict__ M,
                                                                    const float* __restrict__ bias,
                                                                    float* __restrict__ y)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)g.K * g.P) return;
    const int kk = (int)(idx / g.P);
    const int p = (int)(idx % g.P);
    const int tx = p % g.tw;
    const int t2 = p / g.tw;
    const int ty = t2 % g.th;
    const int img = t2 / g.th;
    const long long plane = (long long)g.K * g.ldp;
    const float* mp = M + (long long)kk * g.ldp + p;
    float m[AH][AW];
#pragma unroll
    for (int a = 0; a < AH; ++a)
#pragma unroll
        for (int b = 0; b < AW; ++b) m[a][b] = mp[(long long)(a * AW + b) * plane];
    float t[NH][AW];                     // t = A_h^T m
#pragma unroll
    for (int i = 0; i < NH; ++i)
#pragma unroll
        for (int b = 0; b < AW; ++b) {
            float acc = 0.f;
#pragma unroll
            for (int a = 0; a < AH; ++a) acc = fmaf(ah.v[i][a], m[a][b], acc);
            t[i][b] = acc;
        }
    const float bv = bias ? bias[kk] : 0.f;
    float* yp = y + ((long long)img * g.K + kk) * g.Ho * g.Wo;
#pragma unroll
    for (int i = 0; i < NH; ++i) {
        const int oy = ty * NH + i;
        if (oy >= g.Ho) continue;
#pragma unroll
        for (int j = 0; j < NW; ++j) {
            const int ox = tx * NW + j;
            float acc = bv;
#pragma unroll
            for (int b = 0; b < AW; ++b) acc = fmaf(t[i][b], aw.v[j][b], acc);
            if (ox < g.Wo) yp[(long long)oy * g.Wo + ox] = acc;
        }
    }
}

template <int R, int C>
MatArg<R, C> mat_arg(const float* src)
{
    MatArg<R, C> m;
    for (int i = 0; i < R; ++i)
        for (int j = 0; j < C; ++j) m.v[i][j] = src[i * C + j];
    return m;
}

template <int AH, int AW>
hipError_t launch_input_r(const WinoGeom& g, const float* BTh, const float* BTw, const float* x, float* V, hipStream_t s)
{
    const long long total = (long long)g.C * g.P;
    hipLaunchKernelGGL((input_transform_rect_kernel<AH, AW>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, g,
                       mat_arg<AH, AH>(BTh), mat_arg<AW, AW>(BTw), x, V);
    return hipGetLastError();
}

template <int NH, int NW, int AH, int AW>
hipError_t launch_output_r(const WinoGeom& g, const float* ATh, const float* ATw, const float* M, const float* bias,
                           float* y, hipStream_t s)
{
    const long long total = (long long)g.K * g.P;
    hipLaunchKernelGGL((output_transform_rect_kernel<NH, NW, AH, AW>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       s, g, mat_arg<NH, AH>(ATh), mat_arg<NW, AW>(ATw), M, bias, y);
    return hipGetLastError();
}

bool axis_ok(int n, int k, int alpha)
{
    if (k == 1) return n == 1 && alpha == 1;
    return n >= 2 && n <= 8 && k >= 2 && k <= kMaxK && alpha == n + k - 1 && alpha <= kMaxAlphaT;
}

bool rect_geom_ok(const WinoGeom& g)
{
    if (g.N <= 0 || g.C <= 0 || g.H <= 0 || g.W <= 0 || g.K <= 0 || g.blocked) return false;
    if (!axis_ok(g.n, g.k, g.alpha) || !axis_ok(g.nw, g.kw, g.alpha_w)) return false;
    if (g.k == g.kw) return false;                                // square kernels take the other kernels
    if (g.k > 1 && g.kw > 1 && (g.n != g.nw || g.alpha > kMaxMixedAlpha || g.alpha_w > kMaxMixedAlpha)) return false;
    if (g.Ho != g.H + 2 * g.pad_h - g.k + 1 || g.Wo != g.W + 2 * g.pad_w - g.kw + 1 || g.Ho <= 0 || g.Wo <= 0) return false;
    if (g.th != (g.Ho + g.n - 1) / g.n || g.tw != (g.Wo + g.nw - 1) / g.nw) return false;
    if ((long long)g.P != (long long)g.N * g.th * g.tw) return false;
    if (g.ldp < g.P || g.ldk < g.K) return false;
    if ((long long)g.C * g.ldp >= (1ll << 31) || (long long)g.K * g.ldp >= (1ll << 31)) return false;
    if ((long long)g.H * g.W >= (1ll << 31)) return false;
    return true;
}

}  // namespace

bool winograd_rect_kernels_available(int nh, int kh, int nw, int kw)
{
    if (!axis_ok(nh, kh, nh + kh - 1) || !axis_ok(nw, kw, nw + kw - 1) || kh == kw) return false;
    if (kh > 1 && kw > 1) return nh == nw && nh + kh - 1 <= kMaxMixedAlpha && nw + kw - 1 <= kMaxMixedAlpha;
    return true;
}

hipError_t launch_filter_transform_rect(const WinoGeom& g, const float* Gh, const float* Gw, const float* w, float* U,
                                        hipStream_t s)
{
    if (!rect_geom_ok(g) || !Gh || !Gw || !w || !U) return hipErrorInvalidValue;
    RectFilterMat m;
    for (int i = 0; i < kMaxAlphaT; ++i)
        for (int j = 0; j < kMaxK; ++j) {
            m.gh[i][j] = (i < g.alpha && j < g.k) ? Gh[i * g.k + j] : 0.f;
            m.gw[i][j] = (i < g.alpha_w && j < g.kw) ? Gw[i * g.kw + j] : 0.f;
        }
    const long long total = (long long)g.K * g.C;
    hipLaunchKernelGGL(filter_transform_rect_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, g, m, w, U);
    return hipGetLastError();
}

hipError_t launch_input_transform_rect(const WinoGeom& g, const float* BTh, const float* BTw, const float* x, float* V,
                                       hipStream_t s)
{
    if (!rect_geom_ok(g) || !BTh || !BTw || !x || !V) return hipErrorInvalidValue;
#define MNN_CASE(A)                                                                  \
    if (g.alpha == 1 && g.alpha_w == A) return launch_input_r<1, A>(g, BTh, BTw, x, V, s); \
    if (g.alpha == A && g.alpha_w == 1) return launch_input_r<A, 1>(g, BTh, BTw, x, V, s);
    MNN_CASE(3) MNN_CASE(4) MNN_CASE(5) MNN_CASE(6) MNN_CASE(7) MNN_CASE(8) MNN_CASE(9) MNN_CASE(10)
#undef MNN_CASE
    // several taps on both axes: every pair of different alphas from 3 to 8
    if (g.alpha == 3 && g.alpha_w == 4) return launch_input_r<3, 4>(g, BTh, BTw, x, V, s);
    if (g.alpha == 3 && g.alpha_w == 5) return launch_input_r<3, 5>(g, BTh, BTw, x, V, s);
    if (g.alpha == 3 && g.alpha_w == 6) return launch_input_r<3, 6>(g, BTh, BTw, x, V, s);
    if (g.alpha == 3 && g.alpha_w == 7) return launch_input_r<3, 7>(g, BTh, BTw, x, V, s);
    if (g.alpha == 3 && g.alpha_w == 8) return launch_input_r<3, 8>(g, BTh, BTw, x, V, s);
    if (g.alpha == 4 && g.alpha_w == 3) return launch_input_r<4, 3>(g, BTh, BTw, x, V, s);
    if (g.alpha == 4 && g.alpha_w == 5) return launch_input_r<4, 5>(g, BTh, BTw, x, V, s);
    if (g.alpha == 4 && g.alpha_w == 6) return launch_input_r<4, 6>(g, BTh, BTw, x, V, s);
    if (g.alpha == 4 && g.alpha_w == 7) return launch_input_r<4, 7>(g, BTh, BTw, x, V, s);
    if (g.alpha == 4 && g.alpha_w == 8) return launch_input_r<4, 8>(g, BTh, BTw, x, V, s);
    if (g.alpha == 5 && g.alpha_w == 3) return launch_input_r<5, 3>(g, BTh, BTw, x, V, s);
    if (g.alpha == 5 && g.alpha_w == 4) return launch_input_r<5, 4>(g, BTh, BTw, x, V, s);
    if (g.alpha == 5 && g.alpha_w == 6) return launch_input_r<5, 6>(g, BTh, BTw, x, V, s);
    if (g.alpha == 5 && g.alpha_w == 7) return launch_input_r<5, 7>(g, BTh, BTw, x, V, s);
    if (g.alpha == 5 && g.alpha_w == 8) return launch_input_r<5, 8>(g, BTh, BTw, x, V, s);
    if (g.alpha == 6 && g.alpha_w == 3) return launch_input_r<6, 3>(g, BTh, BTw, x, V, s);
    if (g.alpha == 6 && g.alpha_w == 4) return launch_input_r<6, 4>(g, BTh, BTw, x, V, s);
    if (g.alpha == 6 && g.alpha_w == 5) return launch_input_r<6, 5>(g, BTh, BTw, x, V, s);
    if (g.alpha == 6 && g.alpha_w == 7) return launch_input_r<6, 7>(g, BTh, BTw, x, V, s);
    if (g.alpha == 6 && g.alpha_w == 8) return launch_input_r<6, 8>(g, BTh, BTw, x, V, s);
    if (g.alpha == 7 && g.alpha_w == 3) return launch_input_r<7, 3>(g, BTh, BTw, x, V, s);
    if (g.alpha == 7 && g.alpha_w == 4) return launch_input_r<7, 4>(g, BTh, BTw, x, V, s);
    if (g.alpha == 7 && g.alpha_w == 5) return launch_input_r<7, 5>(g, BTh, BTw, x, V, s);
    if (g.alpha == 7 && g.alpha_w == 6) return launch_input_r<7, 6>(g, BTh, BTw, x, V, s);
    if (g.alpha == 7 && g.alpha_w == 8) return launch_input_r<7, 8>(g, BTh, BTw, x, V, s);
    if (g.alpha == 8 && g.alpha_w == 3) return launch_input_r<8, 3>(g, BTh, BTw, x, V, s);
    if (g.alpha == 8 && g.alpha_w == 4) return launch_input_r<8, 4>(g, BTh, BTw, x, V, s);
    if (g.alpha == 8 && g.alpha_w == 5) return launch_input_r<8, 5>(g, BTh, BTw, x, V, s);
    if (g.alpha == 8 && g.alpha_w == 6) return launch_input_r<8, 6>(g, BTh, BTw, x, V, s);
    if (g.alpha == 8 && g.alpha_w == 7) return launch_input_r<8, 7>(g, BTh, BTw, x, V, s);
    return hipErrorInvalidValue;
}

hipError_t launch_output_transform_rect(const WinoGeom& g, const float* ATh, const float* ATw, const float* M,
                                        const float* bias, float* y, hipStream_t s)
{
    if (!rect_geom_ok(g) || !ATh || !ATw || !M || !y) return hipErrorInvalidValue;
    if (g.k > 1 && g.kw > 1) {
        // n x n tiles of a k_h x k_w kernel: every (n, k_h, k_w) with both alphas up to 8
        if (g.n == 2 && g.k == 2 && g.kw == 3) return launch_output_r<2, 2, 3, 4>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 2 && g.kw == 3) return launch_output_r<3, 3, 4, 5>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 4 && g.k == 2 && g.kw == 3) return launch_output_r<4, 4, 5, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 5 && g.k == 2 && g.kw == 3) return launch_output_r<5, 5, 6, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 6 && g.k == 2 && g.kw == 3) return launch_output_r<6, 6, 7, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 2 && g.kw == 4) return launch_output_r<2, 2, 3, 5>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 2 && g.kw == 4) return launch_output_r<3, 3, 4, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 4 && g.k == 2 && g.kw == 4) return launch_output_r<4, 4, 5, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 5 && g.k == 2 && g.kw == 4) return launch_output_r<5, 5, 6, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 2 && g.kw == 5) return launch_output_r<2, 2, 3, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 2 && g.kw == 5) return launch_output_r<3, 3, 4, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 4 && g.k == 2 && g.kw == 5) return launch_output_r<4, 4, 5, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 2 && g.kw == 6) return launch_output_r<2, 2, 3, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 2 && g.kw == 6) return launch_output_r<3, 3, 4, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 2 && g.kw == 7) return launch_output_r<2, 2, 3, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 3 && g.kw == 2) return launch_output_r<2, 2, 4, 3>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 3 && g.kw == 2) return launch_output_r<3, 3, 5, 4>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 4 && g.k == 3 && g.kw == 2) return launch_output_r<4, 4, 6, 5>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 5 && g.k == 3 && g.kw == 2) return launch_output_r<5, 5, 7, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 6 && g.k == 3 && g.kw == 2) return launch_output_r<6, 6, 8, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 3 && g.kw == 4) return launch_output_r<2, 2, 4, 5>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 3 && g.kw == 4) return launch_output_r<3, 3, 5, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 4 && g.k == 3 && g.kw == 4) return launch_output_r<4, 4, 6, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 5 && g.k == 3 && g.kw == 4) return launch_output_r<5, 5, 7, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 3 && g.kw == 5) return launch_output_r<2, 2, 4, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 3 && g.kw == 5) return launch_output_r<3, 3, 5, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 4 && g.k == 3 && g.kw == 5) return launch_output_r<4, 4, 6, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 3 && g.kw == 6) return launch_output_r<2, 2, 4, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 3 && g.kw == 6) return launch_output_r<3, 3, 5, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 3 && g.kw == 7) return launch_output_r<2, 2, 4, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 4 && g.kw == 2) return launch_output_r<2, 2, 5, 3>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 4 && g.kw == 2) return launch_output_r<3, 3, 6, 4>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 4 && g.k == 4 && g.kw == 2) return launch_output_r<4, 4, 7, 5>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 5 && g.k == 4 && g.kw == 2) return launch_output_r<5, 5, 8, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 4 && g.kw == 3) return launch_output_r<2, 2, 5, 4>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 4 && g.kw == 3) return launch_output_r<3, 3, 6, 5>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 4 && g.k == 4 && g.kw == 3) return launch_output_r<4, 4, 7, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 5 && g.k == 4 && g.kw == 3) return launch_output_r<5, 5, 8, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 4 && g.kw == 5) return launch_output_r<2, 2, 5, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 4 && g.kw == 5) return launch_output_r<3, 3, 6, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 4 && g.k == 4 && g.kw == 5) return launch_output_r<4, 4, 7, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 4 && g.kw == 6) return launch_output_r<2, 2, 5, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 4 && g.kw == 6) return launch_output_r<3, 3, 6, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 4 && g.kw == 7) return launch_output_r<2, 2, 5, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 5 && g.kw == 2) return launch_output_r<2, 2, 6, 3>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 5 && g.kw == 2) return launch_output_r<3, 3, 7, 4>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 4 && g.k == 5 && g.kw == 2) return launch_output_r<4, 4, 8, 5>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 5 && g.kw == 3) return launch_output_r<2, 2, 6, 4>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 5 && g.kw == 3) return launch_output_r<3, 3, 7, 5>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 4 && g.k == 5 && g.kw == 3) return launch_output_r<4, 4, 8, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 5 && g.kw == 4) return launch_output_r<2, 2, 6, 5>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 5 && g.kw == 4) return launch_output_r<3, 3, 7, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 4 && g.k == 5 && g.kw == 4) return launch_output_r<4, 4, 8, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 5 && g.kw == 6) return launch_output_r<2, 2, 6, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 5 && g.kw == 6) return launch_output_r<3, 3, 7, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 5 && g.kw == 7) return launch_output_r<2, 2, 6, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 6 && g.kw == 2) return launch_output_r<2, 2, 7, 3>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 6 && g.kw == 2) return launch_output_r<3, 3, 8, 4>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 6 && g.kw == 3) return launch_output_r<2, 2, 7, 4>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 6 && g.kw == 3) return launch_output_r<3, 3, 8, 5>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 6 && g.kw == 4) return launch_output_r<2, 2, 7, 5>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 6 && g.kw == 4) return launch_output_r<3, 3, 8, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 6 && g.kw == 5) return launch_output_r<2, 2, 7, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 3 && g.k == 6 && g.kw == 5) return launch_output_r<3, 3, 8, 7>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 6 && g.kw == 7) return launch_output_r<2, 2, 7, 8>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 7 && g.kw == 2) return launch_output_r<2, 2, 8, 3>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 7 && g.kw == 3) return launch_output_r<2, 2, 8, 4>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 7 && g.kw == 4) return launch_output_r<2, 2, 8, 5>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 7 && g.kw == 5) return launch_output_r<2, 2, 8, 6>(g, ATh, ATw, M, bias, y, s);
        if (g.n == 2 && g.k == 7 && g.kw == 6) return launch_output_r<2, 2, 8, 7>(g, ATh, ATw, M, bias, y, s);
        return hipErrorInvalidValue;
    }
    const int n = g.k == 1 ? g.nw : g.n, k = g.k == 1 ? g.kw : g.k;
#define MNN_NK(NN, KK)                                                                                       \
    if (n == NN && k == KK) {                                                                                \
        if (g.k == 1) return launch_output_r<1, NN, 1, NN + KK - 1>(g, ATh, ATw, M, bias, y, s);             \
        return launch_output_r<NN, 1, NN + KK - 1, 1>(g, ATh, ATw, M, bias, y, s);                           \
    }
    // every (n, k) with 2 <= n <= 8, 2 <= k <= 7 and n + k - 1 <= 10
    MNN_NK(2, 2) MNN_NK(3, 2) MNN_NK(4, 2) MNN_NK(5, 2) MNN_NK(6, 2) MNN_NK(7, 2) MNN_NK(8, 2)
    MNN_NK(2, 3) MNN_NK(3, 3) MNN_NK(4, 3) MNN_NK(5, 3) MNN_NK(6, 3) MNN_NK(7, 3) MNN_NK(8, 3)
    MNN_NK(2, 4) MNN_NK(3, 4) MNN_NK(4, 4) MNN_NK(5, 4) MNN_NK(6, 4) MNN_NK(7, 4)
    MNN_NK(2, 5) MNN_NK(3, 5) MNN_NK(4, 5) MNN_NK(5, 5) MNN_NK(6, 5)
    MNN_NK(2, 6) MNN_NK(3, 6) MNN_NK(4, 6) MNN_NK(5, 6)
    MNN_NK(2, 7) MNN_NK(3, 7) MNN_NK(4, 7)
#undef MNN_NK
    return hipErrorInvalidValue;
}

}  // namespace mnnconv
