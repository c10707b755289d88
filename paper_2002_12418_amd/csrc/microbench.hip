// Two device-rate probes behind the roofline figures: how fast this GPU issues fp32 matrix-core instructions
// when nothing else is in the way, and how fast a plain kernel streams memory.  They measure the "known
// constants for a specific backend" of Section 3.2 (2) of the MNN paper (FLOPS, and the memory rate next to
// it) at their upper limits; the cost model itself uses the rates the library's own kernels reach.
//
//   * mfma_issue_kernel: every wave issues v_mfma_f32_32x32x2_f32 back to back on four independent
//     accumulators held in registers (no memory access inside the loop).  One instruction is 32*32*2
//     multiply-adds; the result is written once at the end so that the loop cannot be dropped.
//   * stream_copy_kernel: one 16-byte load and store per lane, one workgroup per 4 KiB (a grid of short workgroups
//     in address order streams faster on this part than a grid-stride loop: 6.2 against 4.6 - 5.1 TB/s).
#include <hip/hip_runtime.h>
#include "kernels.hpp"

namespace mnnconv {
namespace {

using float16v = __attribute__((ext_vector_type(16))) float;

__global__ __launch_bounds__(256) void mfma_issue_kernel(float* __restrict__ out, int iters, float seed)
{
    float16v acc0 = {}, acc1 = {}, acc2 = {}, acc3 = {};
    const float a = seed * (float)(threadIdx.x & 63), b = seed * (float)((threadIdx.x >> 2) + 1);
    for (int i = 0; i < iters; ++i) {
        acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, a, acc1, 0, 0, 0);
        acc2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, a, acc2, 0, 0, 0);
        acc3 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, b, acc3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 16; ++j) s += (acc0[j] + acc1[j]) + (acc2[j] + acc3[j]);
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const float4* __restrict__ src, float4* __restrict__ dst, size_t n4)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n4) dst[i] = src[i];
}

}  // namespace

hipError_t launch_mfma_issue(float* out, int workgroups, int iters, hipStream_t s)
{
    if (!out || workgroups <= 0 || iters <= 0) return hipErrorInvalidValue;
    mfma_issue_kernel<<<workgroups, 256, 0, s>>>(out, iters, 1e-3f);
    return hipGetLastError();
}

hipError_t launch_stream_copy(const float* src, float* dst, size_t n_floats, hipStream_t s)
{
    if (!src || !dst || (n_floats & 3) || (((uintptr_t)src | (uintptr_t)dst) & 15)) return hipErrorInvalidValue;
    if (n_floats == 0) return hipSuccess;
    const size_t n4 = n_floats / 4, blocks = (n4 + 255) / 256;
    if (blocks >= (1ull << 31)) return hipErrorInvalidValue;
    stream_copy_kernel<<<(unsigned)blocks, 256, 0, s>>>((const float4*)src, (float4*)dst, n4);
    return hipGetLastError();
}

}  // namespace mnnconv
