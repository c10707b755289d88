// Device-memory fills that the host side needs where a runtime memset will not do.
//
//   * fill_pattern: seeded, reproducible pseudo-random floats in [lo, hi].  The pre-inference step of Section 3.2 of
//     the MNN paper times candidate schemes on scratch tensors; on this GPU the power a matrix-core instruction
//     draws, and with it the clock the chip sustains, depends on how many operand bits toggle, so timing on
//     all-zero tensors rates the matrix-multiplication stage a few per cent faster than inference on real
//     activations will see it.  Candidates are therefore timed on this pattern.
//   * fill_zero: zeros written by a kernel.  A memset node recorded into a HIP graph is not reliable on this
//     platform; code that a caller may capture clears memory with this kernel instead.
#include <hip/hip_runtime.h>
#include "kernels.hpp"

namespace mnnconv {
namespace {

// one round of a 32-bit integer hash (multiply-xorshift): every index gets an independent-looking word
__device__ __forceinline__ unsigned mix32(unsigned v)
{
    v ^= v >> 16; v *= 0x7feb352du;
    v ^= v >> 15; v *= 0x846ca68bu;
    v ^= v >> 16;
    return v;
}

__global__ __launch_bounds__(256) void fill_pattern_kernel(float* __restrict__ dst, size_t n, unsigned seed, float lo, float scale)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const unsigned h = mix32((unsigned)i * 0x9e3779b9u + (unsigned)(i >> 32) + seed);
    dst[i] = lo + scale * (float)(h >> 8);          // 24 random bits
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float4* __restrict__ dst4, size_t n4, float* __restrict__ tail, int ntail)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) dst4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < (size_t)ntail) tail[i] = 0.f;
}

}  // namespace

hipError_t launch_fill_pattern(float* dst, size_t n_floats, unsigned seed, float lo, float hi, hipStream_t s)
{
    if (!dst || !(hi >= lo)) return hipErrorInvalidValue;
    if (n_floats == 0) return hipSuccess;
    const size_t blocks = (n_floats + 255) / 256;
    if (blocks >= (1ull << 31)) return hipErrorInvalidValue;
    fill_pattern_kernel<<<(unsigned)blocks, 256, 0, s>>>(dst, n_floats, seed, lo, (hi - lo) / 16777215.f);
    return hipGetLastError();
}

hipError_t launch_fill_zero(float* dst, size_t n_floats, hipStream_t s)
{
    if (!dst || ((uintptr_t)dst & 15)) return hipErrorInvalidValue;      // 16-byte aligned base
    if (n_floats == 0) return hipSuccess;
    const size_t n4 = n_floats / 4;
    const int ntail = (int)(n_floats & 3);
    const size_t blocks = (n4 + 255) / 256 + (n4 == 0 ? 1 : 0);
    if (blocks >= (1ull << 31)) return hipErrorInvalidValue;
    fill_zero_kernel<<<(unsigned)blocks, 256, 0, s>>>((float4*)dst, n4, dst + n4 * 4, ntail);
    return hipGetLastError();
}

}  // namespace mnnconv
