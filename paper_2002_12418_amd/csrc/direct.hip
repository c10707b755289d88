// Sliding-window convolution (the scheme Section 3.2 (1) of the MNN paper falls
// back to when Winograd does not pay off, and the only scheme for strided or
// dilated layers) and the weight re-layout used by the GEMM paths.
#include <hip/hip_runtime.h>
#include "kernels.hpp"

namespace mnnconv {
namespace {

// One lane per output element; consecutive lanes walk along W_o so that input
// reads of a wavefront are contiguous (stride 1) or evenly strided, and weight
// reads are wave-uniform (scalar loads).
__global__ __launch_bounds__(256) void direct_conv_kernel(DirectGeom g, const float* __restrict__ x,
                                                          const float* __restrict__ w,
                                                          const float* __restrict__ bias,
                                                          float* __restrict__ y)
{
    const int plane = g.Ho * g.Wo;
    const int pix = blockIdx.x * 256 + threadIdx.x;
    const int kk = blockIdx.y;
    const int img = blockIdx.z;
    if (pix >= plane) return;
    const int oy = pix / g.Wo, ox = pix % g.Wo;
    const int iy0 = oy * g.stride_h - g.pad_h;
    const int ix0 = ox * g.stride_w - g.pad_w;
    const float* xi = x + (long long)img * g.C * g.H * g.W;
    const float* wk = w + (long long)kk * g.C * g.kh * g.kw;
    float acc = 0.f;
    for (int c = 0; c < g.C; ++c) {
        const float* xc = xi + (long long)c * g.H * g.W;
        const float* wc = wk + (long long)c * g.kh * g.kw;
        for (int r = 0; r < g.kh; ++r) {
            const int iy = iy0 + r * g.dil_h;
            if (iy < 0 || iy >= g.H) continue;
            for (int s = 0; s < g.kw; ++s) {
                const int ix = ix0 + s * g.dil_w;
                if (ix < 0 || ix >= g.W) continue;
                acc = fmaf(xc[(long long)iy * g.W + ix], wc[r * g.kw + s], acc);
            }
        }
    }
    if (bias) acc += bias[kk];
    y[((long long)img * g.K + kk) * plane + pix] = acc;
}

__global__ __launch_bounds__(256) void weight_transpose_kernel(const float* __restrict__ w, float* __restrict__ Wt,
                                                               int K, int R, int ldk)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)R * ldk) return;
    const int kk = (int)(idx % ldk);
    const int r = (int)(idx / ldk);
    Wt[idx] = (kk < K) ? w[(long long)kk * R + r] : 0.f;
}

}  // namespace

hipError_t launch_direct_conv(const DirectGeom& g, const float* x, const float* w, const float* bias, float* y,
                              hipStream_t s)
{
    if (!x || !w || !y) return hipErrorInvalidValue;
    if (g.N <= 0 || g.C <= 0 || g.H <= 0 || g.W <= 0 || g.K <= 0 || g.kh <= 0 || g.kw <= 0) return hipErrorInvalidValue;
    if (g.Ho <= 0 || g.Wo <= 0 || g.stride_h <= 0 || g.stride_w <= 0 || g.dil_h <= 0 || g.dil_w <= 0)
        return hipErrorInvalidValue;
    if ((long long)g.Ho * g.Wo >= (1ll << 31) || g.K > 65535 || g.N > 65535) return hipErrorInvalidValue;
    const unsigned bx = (unsigned)(((long long)g.Ho * g.Wo + 255) / 256);
    hipLaunchKernelGGL(direct_conv_kernel, dim3(bx, (unsigned)g.K, (unsigned)g.N), dim3(256), 0, s, g, x, w, bias, y);
    return hipGetLastError();
}

hipError_t launch_weight_transpose(const float* w, float* Wt, int K, int R, int ldk, hipStream_t s)
{
    if (!w || !Wt || K <= 0 || R <= 0 || ldk < K) return hipErrorInvalidValue;
    const long long total = (long long)R * ldk;
    hipLaunchKernelGGL(weight_transpose_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w, Wt, K, R,
                       ldk);
    return hipGetLastError();
}

}  // namespace mnnconv
