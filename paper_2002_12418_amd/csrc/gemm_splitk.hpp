// Split-K for GEMMs with too few output tiles to fill 256 CUs (batch-1 layers: a 512 x 49 output is 8
// tiles however long its reduction is).  The reduction range of a tile is cut into `splitk` slices, one
// workgroup each.  Every workgroup parks its partial accumulators in a scratch buffer; the one that
// arrives last at the tile's counter adds the slices up in slice order, so the result does not depend on
// arrival order (two runs give the same bits), applies the bias and stores the tile.  The counter is reset
// by that workgroup, so the buffers need no clearing between launches.
#pragma once
#include <hip/hip_runtime.h>

namespace mnnconv {

typedef float splitk_floatx16 __attribute__((ext_vector_type(16)));

// Returns true in the workgroup that must write the tile; its acc then holds the full sum.
// partial: [tile][split][TM*TN*16][NT] floats, counters: [tile] (zero before the first launch).
template <int TM, int TN, int NT>
__device__ __forceinline__ bool splitk_combine(splitk_floatx16 (&acc)[TM][TN], float* __restrict__ partial,
                                               unsigned* __restrict__ counters, int tile, int split, int splitk, int tid)
{
    constexpr int REGS = TM * TN * 16;
    float* mine = partial + ((long long)tile * splitk + split) * REGS * NT + tid;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[((i * TN + j) * 16 + r) * NT] = acc[i][j][r];
    __threadfence();                               // partials visible device-wide before the arrival is counted
    __shared__ unsigned arrived;
    __syncthreads();
    if (tid == 0) arrived = atomicAdd(&counters[tile], 1u);
    __syncthreads();
    if (arrived != (unsigned)(splitk - 1)) return false;
    __threadfence();
    const float* base = partial + (long long)tile * splitk * REGS * NT + tid;
    // Slice by slice, so that every element is summed in slice order whoever arrived when; the 16 loads of
    // a slice (and of the next three) are independent and in flight together.
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const float* blk = base + (long long)((i * TN + j) * 16) * NT;
            splitk_floatx16 s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.f;
            int sl = 0;
            for (; sl + 4 <= splitk; sl += 4) {
                float v[4][16];
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        v[q][r] = __builtin_nontemporal_load(blk + ((long long)(sl + q) * REGS + r) * NT);
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int r = 0; r < 16; ++r) s[r] += v[q][r];
            }
            for (; sl < splitk; ++sl) {
                float v[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) v[r] = __builtin_nontemporal_load(blk + ((long long)sl * REGS + r) * NT);
#pragma unroll
                for (int r = 0; r < 16; ++r) s[r] += v[r];
            }
            acc[i][j] = s;
        }
    if (tid == 0) counters[tile] = 0u;             // ready for the next launch
    return true;
}

}  // namespace mnnconv
