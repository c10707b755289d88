// Result stores of the matrix-core GEMM kernels (32x32 accumulator tiles) and split-K.
//
// Split-K: a GEMM with too few output tiles to fill 256 CUs (batch-1 layers: a 512 x 49 output is 8 tiles
// however long its reduction is) cuts the reduction of every tile into `splitk` slices, one workgroup each.
// Every workgroup writes its partial tile to slice `split` of a scratch tensor P[split][batch][M][ldc];
// a second kernel adds the slices in slice order, applies the bias and writes the result.  The order of
// the additions is fixed, so two runs give the same bits, and the only synchronisation is the kernel
// boundary: a device-wide fence inside the GEMM kernel (the one-kernel alternative) makes every
// workgroup wait for an L2 write-back on this multi-die part and costs more than the second launch.
#pragma once
#include <hip/hip_runtime.h>
#include "kernels.hpp"

namespace mnnconv {

constexpr int kStageStride = 36;      // floats per row of a wavefront's 32x32 staging tile in LDS
constexpr int kStageFloats = 32 * kStageStride;

// element (m, col) of the destination lives at base + (col / L) * sImg + m * sRow + col % L
struct TileDest { float* base; long long sImg, sRow; int L; const float* bias; };

__device__ __forceinline__ TileDest tile_dest(const GemmProblem& p, int b, int split, int splitk, int ldc)
{
    if (splitk > 1)
        return TileDest{p.splitk_partial + ((long long)split * p.batch + b) * p.M * ldc, 0, ldc, ldc, nullptr};
    return TileDest{p.D + (long long)b * p.strideD_batch, p.strideD_img, p.strideD_row, p.L, p.bias};
}

// Stores the TM x TN accumulator tiles of one wavefront whose block starts at row mw0, column nw0.
// Accumulator layout of v_mfma_f32_32x32x*: lane l holds column l % 32, rows 8*(r/4) + 4*(l/32) + r%4.
// vec != 0 (16-byte aligned destination rows, 4 | L, 4 | Ncols): through `stage`, a wavefront-private LDS
// tile, so that a lane stores 4 consecutive columns of one row and one store instruction covers 8 rows x
// 128 bytes instead of 2 rows x 128 bytes in 4-byte pieces.  LDS accesses of one wavefront execute in
// order, so the staging needs no barrier (the caller's LDS must be free: after its last barrier).
template <int TM, int TN, typename Acc>
__device__ __forceinline__ void store_tiles(const Acc (&acc)[TM][TN], const TileDest& d, int M, int Ncols, int mw0,
                                            int nw0, int lane, float* stage, int vec)
{
    const int lrow = lane >> 5, lcol = lane & 31;
    if (vec) {
        const int rrow = lane >> 3, rc4 = (lane & 7) * 4;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = nw0 + j * 32 + rc4;
            const bool cok = col < Ncols;                     // 4 | Ncols: all four columns or none
            const long long coff = (long long)(col / d.L) * d.sImg + (col % d.L);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    stage[(8 * (r / 4) + 4 * lrow + (r % 4)) * kStageStride + lcol] = acc[i][j][r];
#pragma unroll
                for (int ps = 0; ps < 4; ++ps) {
                    const int row = ps * 8 + rrow;
                    const int m = mw0 + i * 32 + row;
                    float4 v = *reinterpret_cast<const float4*>(&stage[row * kStageStride + rc4]);
                    if (cok && m < M) {
                        if (d.bias) {
                            const float bv = d.bias[m];
                            v.x += bv; v.y += bv; v.z += bv; v.w += bv;
                        }
                        *reinterpret_cast<float4*>(d.base + coff + (long long)m * d.sRow) = v;
                    }
                }
            }
        }
        return;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = nw0 + j * 32 + lcol;
        if (col >= Ncols) continue;
        const long long coff = (long long)(col / d.L) * d.sImg + (col % d.L);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mbase = mw0 + i * 32 + 4 * lrow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = mbase + 8 * (r / 4) + (r % 4);
                if (m < M) {
                    float v = acc[i][j][r];
                    if (d.bias) v += d.bias[m];
                    d.base[coff + (long long)m * d.sRow] = v;
                }
            }
        }
    }
}

// whether the result rows of `p` (or of its split-K scratch tensor) can take 16-byte stores
inline int result_rows_vectorisable(const GemmProblem& p)
{
    if (p.Ncols % 4 != 0) return 0;
    if (p.splitk > 1) return (reinterpret_cast<uintptr_t>(p.splitk_partial) & 15u) == 0 ? 1 : 0;
    return ((reinterpret_cast<uintptr_t>(p.D) & 15u) == 0 && p.L % 4 == 0 && p.strideD_batch % 4 == 0 &&
            p.strideD_img % 4 == 0 && p.strideD_row % 4 == 0) ? 1 : 0;
}

}  // namespace mnnconv
