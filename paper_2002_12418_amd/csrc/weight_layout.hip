// Weight re-layout for the GEMM-shaped schemes: the 1x1 convolution (Section 3.2 (1) item 1 of the MNN
// paper) and the sliding-window scheme run as an implicit GEMM.  Both want the weights with the
// reduction index (c, kr, ks) as the slow dimension and the output channel contiguous.
#include <hip/hip_runtime.h>
#include "kernels.hpp"

namespace mnnconv {
namespace {

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

hipError_t launch_weight_transpose(const float* w, float* Wt, int K, int R, int ldk, hipStream_t s)
{
    if (!w || !Wt || K <= 0 || R <= 0 || ldk < K) return hipErrorInvalidValue;
    const long long total = (long long)R * ldk;
    hipLaunchKernelGGL(weight_transpose_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, w, Wt, K, R,
                       ldk);
    return hipGetLastError();
}

}  // namespace mnnconv
