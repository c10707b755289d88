/*
 * CPU oracle: 2-D convolution written out from its definition, in float64.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call or link
 * this file; it shares no code, header, table or helper with the HIP library.
 *
 * What it computes (the result that both the Winograd form, Section 3.3.1
 * Eq. "Y = A^T[ sum_channel (G W G^T) (.) (B^T X B) ] A", and the k = 1
 * matrix-multiplication form, Section 3.2 item (1), reach exactly up to
 * rounding order):
 *
 *   H_o = floor((H + 2*pad_h - dil_h*(kh-1) - 1) / stride_h) + 1     (W_o alike)
 *   y[n,k,oy,ox] = b[k] + sum_{c<C} sum_{r<kh} sum_{s<kw}
 *        xpad[n, c, oy*stride_h - pad_h + r*dil_h, ox*stride_w - pad_w + s*dil_w] * w[k,c,r,s]
 *
 * with xpad equal to x inside [0,H) x [0,W) and 0 outside.  It is a
 * cross-correlation (the kernel is not flipped), which is the form the
 * paper's Winograd identity and the cited fast-convolution work use.
 *
 * Inputs are float32 values widened to float64; all products and sums are
 * float64; the result is returned as float64.  Loops are in the order of the
 * definition; the only parallelism is OpenMP over independent (n,k) planes.
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_conv2d_f64(const float *x, const float *w, const float *b /* may be NULL */,
                      double *y,
                      int64_t N, int64_t C, int64_t H, int64_t W,
                      int64_t K, int64_t kh, int64_t kw,
                      int64_t stride_h, int64_t stride_w,
                      int64_t pad_h, int64_t pad_w,
                      int64_t dil_h, int64_t dil_w)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || kh <= 0 || kw <= 0) return -1;
    if (stride_h <= 0 || stride_w <= 0 || dil_h <= 0 || dil_w <= 0 || pad_h < 0 || pad_w < 0) return -1;
    const int64_t eh = H + 2 * pad_h - dil_h * (kh - 1) - 1;
    const int64_t ew = W + 2 * pad_w - dil_w * (kw - 1) - 1;
    if (eh < 0 || ew < 0) return -2;
    const int64_t Ho = eh / stride_h + 1;
    const int64_t Wo = ew / stride_w + 1;

    const int64_t planes = N * K;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t pl = 0; pl < planes; ++pl) {
        const int64_t n = pl / K, k = pl % K;
        double *yp = y + (size_t)pl * (size_t)(Ho * Wo);
        const double bias = b ? (double)b[k] : 0.0;
        for (int64_t oy = 0; oy < Ho; ++oy) {
            for (int64_t ox = 0; ox < Wo; ++ox) {
                double acc = 0.0;
                for (int64_t c = 0; c < C; ++c) {
                    const float *xc = x + ((size_t)(n * C + c)) * (size_t)(H * W);
                    const float *wc = w + ((size_t)(k * C + c)) * (size_t)(kh * kw);
                    for (int64_t r = 0; r < kh; ++r) {
                        const int64_t iy = oy * stride_h - pad_h + r * dil_h;
                        if (iy < 0 || iy >= H) continue;
                        for (int64_t s = 0; s < kw; ++s) {
                            const int64_t ix = ox * stride_w - pad_w + s * dil_w;
                            if (ix < 0 || ix >= W) continue;
                            acc += (double)xc[iy * W + ix] * (double)wc[r * kw + s];
                        }
                    }
                }
                yp[oy * Wo + ox] = bias + acc;
            }
        }
    }
    return 0;
}

/* Evaluate the same definition at a list of output coordinates only
 * (coords: count x 4 int64 = n,k,oy,ox).  Used to sample very large layers. */
int oracle_conv2d_f64_points(const float *x, const float *w, const float *b,
                             const int64_t *coords, int64_t count, double *out,
                             int64_t N, int64_t C, int64_t H, int64_t W,
                             int64_t K, int64_t kh, int64_t kw,
                             int64_t stride_h, int64_t stride_w,
                             int64_t pad_h, int64_t pad_w,
                             int64_t dil_h, int64_t dil_w)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || kh <= 0 || kw <= 0) return -1;
    if (stride_h <= 0 || stride_w <= 0 || dil_h <= 0 || dil_w <= 0 || pad_h < 0 || pad_w < 0) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const int64_t n = coords[4 * i + 0], k = coords[4 * i + 1];
        const int64_t oy = coords[4 * i + 2], ox = coords[4 * i + 3];
        double acc = 0.0;
        for (int64_t c = 0; c < C; ++c) {
            const float *xc = x + ((size_t)(n * C + c)) * (size_t)(H * W);
            const float *wc = w + ((size_t)(k * C + c)) * (size_t)(kh * kw);
            for (int64_t r = 0; r < kh; ++r) {
                const int64_t iy = oy * stride_h - pad_h + r * dil_h;
                if (iy < 0 || iy >= H) continue;
                for (int64_t s = 0; s < kw; ++s) {
                    const int64_t ix = ox * stride_w - pad_w + s * dil_w;
                    if (ix < 0 || ix >= W) continue;
                    acc += (double)xc[iy * W + ix] * (double)wc[r * kw + s];
                }
            }
        }
        out[i] = (b ? (double)b[k] : 0.0) + acc;
    }
    return 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
