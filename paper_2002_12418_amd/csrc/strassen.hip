// Strassen's algorithm for the large matrix multiplication of Section 3.3.2 of the MNN paper, in the
// 7-product / 15-addition form the paper counts (4 additions on each operand, 7 on the result; the
// Winograd variant of Strassen's scheme), arranged for a GPU:
//
//   * one level turns a product D = A B into 7 products of half size.  Here every level is three launches
//     whatever its depth: an "expand" kernel writes the 7 left (right) operands of all sub-products as one
//     dense batch, ONE batched GEMM multiplies them, a "combine" kernel adds the 7 results into the four
//     quadrants of the parent.  Level l works on a batch of 7^l problems.
//   * the additions are plain streaming kernels (16-byte accesses), bound by HBM; the left operand is the
//     weight matrix in the convolution use, so its expansion runs once per weight set.
//
// A is stored transposed (At[r][m], reduction index slow) as everywhere in this library.  With
//   X11 = X(r < R/2, c < C/2), X12 = X(r < R/2, c >= C/2), X21 = X(r >= R/2, c < C/2), X22
// of a row-major [R][C] operand, the quadrants of A (M x R) are A11 = At11, A12 = At21, A21 = At12, A22 = At22.
//   S1 = A21 + A22   S2 = S1 - A11   S3 = A11 - A21   S4 = A12 - S2
//   T1 = B12 - B11   T2 = B22 - T1   T3 = B22 - B12   T4 = T2 - B21
//   P1 = A11 B11  P2 = A12 B21  P3 = S4 B22  P4 = A22 T4  P5 = S1 T1  P6 = S2 T2  P7 = S3 T3
//   C11 = P1 + P2          U2 = P1 + P6   U3 = U2 + P7   U4 = U2 + P5
//   C12 = U4 + P3          C21 = U3 - P4  C22 = U3 + P5
#include <hip/hip_runtime.h>
#include "kernels.hpp"

namespace mnnconv {
namespace {

__device__ __forceinline__ float4 f4add(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
__device__ __forceinline__ float4 f4sub(float4 a, float4 b) { return make_float4(a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w); }

__device__ __forceinline__ long long view_offset(const StrassenView& v, int r, int c)
{
    return (long long)(c / v.L) * v.sImg + (long long)r * v.sRow + (c % v.L);
}

// src: batch of nb row-major [2*rh][2*ch] operands (view v, batch stride sb); dst: [7*nb][rh][ch] dense.
template <bool LEFT>
__global__ __launch_bounds__(256) void strassen_expand_kernel(StrassenView v, const float* __restrict__ src, long long sb,
                                                              int rh, int ch, int nb, float* __restrict__ dst)
{
    const int q = ch >> 2;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)nb * rh * q) return;
    const int c = (int)(idx % q) * 4;
    const long long t = idx / q;
    const int r = (int)(t % rh), b = (int)(t / rh);
    const float* s = src + (long long)b * sb;
    const float4 x11 = *reinterpret_cast<const float4*>(s + view_offset(v, r, c));
    const float4 x12 = *reinterpret_cast<const float4*>(s + view_offset(v, r, c + ch));
    const float4 x21 = *reinterpret_cast<const float4*>(s + view_offset(v, r + rh, c));
    const float4 x22 = *reinterpret_cast<const float4*>(s + view_offset(v, r + rh, c + ch));
    float4 o[7];
    if (LEFT) {       // A11 = x11, A12 = x21, A21 = x12, A22 = x22
        const float4 s1 = f4add(x12, x22), s2 = f4sub(s1, x11);
        o[0] = x11; o[1] = x21; o[2] = f4sub(x21, s2); o[3] = x22; o[4] = s1; o[5] = s2; o[6] = f4sub(x11, x12);
    } else {          // B11 = x11, B12 = x12, B21 = x21, B22 = x22
        const float4 t1 = f4sub(x12, x11), t2 = f4sub(x22, t1);
        o[0] = x11; o[1] = x21; o[2] = x22; o[3] = f4sub(t2, x21); o[4] = t1; o[5] = t2; o[6] = f4sub(x22, x12);
    }
    const long long plane = (long long)rh * ch;
    float* d = dst + (long long)b * 7 * plane + (long long)r * ch + c;
#pragma unroll
    for (int i = 0; i < 7; ++i) *reinterpret_cast<float4*>(d + i * plane) = o[i];
}

// src: [7*nb][mh][ch] dense products; dst: batch of nb [2*mh][2*ch] results (view v, batch stride db), + bias[m].
__global__ __launch_bounds__(256) void strassen_combine_kernel(StrassenView v, const float* __restrict__ src, int mh, int ch,
                                                               int nb, float* __restrict__ dst, long long db,
                                                               const float* __restrict__ bias)
{
    const int q = ch >> 2;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)nb * mh * q) return;
    const int c = (int)(idx % q) * 4;
    const long long t = idx / q;
    const int m = (int)(t % mh), b = (int)(t / mh);
    const long long plane = (long long)mh * ch;
    const float* s = src + (long long)b * 7 * plane + (long long)m * ch + c;
    float4 p[7];
#pragma unroll
    for (int i = 0; i < 7; ++i) p[i] = *reinterpret_cast<const float4*>(s + i * plane);
    const float4 u2 = f4add(p[0], p[5]), u3 = f4add(u2, p[6]), u4 = f4add(u2, p[4]);
    float4 c11 = f4add(p[0], p[1]), c12 = f4add(u4, p[2]), c21 = f4sub(u3, p[3]), c22 = f4add(u3, p[4]);
    if (bias) {
        const float b0 = bias[m], b1 = bias[m + mh];
        const float4 v0 = make_float4(b0, b0, b0, b0), v1 = make_float4(b1, b1, b1, b1);
        c11 = f4add(c11, v0); c12 = f4add(c12, v0); c21 = f4add(c21, v1); c22 = f4add(c22, v1);
    }
    float* d = dst + (long long)b * db;
    *reinterpret_cast<float4*>(d + view_offset(v, m, c)) = c11;
    *reinterpret_cast<float4*>(d + view_offset(v, m, c + ch)) = c12;
    *reinterpret_cast<float4*>(d + view_offset(v, m + mh, c)) = c21;
    *reinterpret_cast<float4*>(d + view_offset(v, m + mh, c + ch)) = c22;
}

bool view_ok(const StrassenView& v, const void* p, int cols_half)
{
    return p && v.L > 0 && v.L % 4 == 0 && v.sImg % 4 == 0 && v.sRow % 4 == 0 && cols_half > 0 && cols_half % 4 == 0 &&
           (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
}

}  // namespace

hipError_t launch_strassen_expand(bool left, const StrassenView& v, const float* src, long long src_batch_stride, int rows_half,
                                  int cols_half, int nb, float* dst, hipStream_t s)
{
    if (!view_ok(v, src, cols_half) || !dst || rows_half <= 0 || nb <= 0 || (src_batch_stride & 3)) return hipErrorInvalidValue;
    const long long total = (long long)nb * rows_half * (cols_half / 4);
    if ((total + 255) / 256 >= (1ll << 31)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (left)
        hipLaunchKernelGGL(strassen_expand_kernel<true>, grid, dim3(256), 0, s, v, src, src_batch_stride, rows_half, cols_half, nb, dst);
    else
        hipLaunchKernelGGL(strassen_expand_kernel<false>, grid, dim3(256), 0, s, v, src, src_batch_stride, rows_half, cols_half, nb, dst);
    return hipGetLastError();
}

hipError_t launch_strassen_combine(const StrassenView& v, const float* src, int rows_half, int cols_half, int nb, float* dst,
                                   long long dst_batch_stride, const float* bias, hipStream_t s)
{
    if (!view_ok(v, dst, cols_half) || !src || rows_half <= 0 || nb <= 0 || (dst_batch_stride & 3)) return hipErrorInvalidValue;
    const long long total = (long long)nb * rows_half * (cols_half / 4);
    if ((total + 255) / 256 >= (1ll << 31)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(strassen_combine_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, v, src, rows_half,
                       cols_half, nb, dst, dst_batch_stride, bias);
    return hipGetLastError();
}

}  // namespace mnnconv
