// Batched GEMM with bf16 matrix-core operands and fp32 accumulation for gfx950
// (v_mfma_f32_32x32x16_bf16), fed from the same fp32 tensors as the fp32 kernel:
//
//   D_b[m][col] = sum_r At_b[r][m] * B_b[r][col] (+ bias[m])
//
// fp32 MFMA on this chip runs at 1/16 of the bf16 rate, so the Winograd-domain
// products (Section 3.3.1 (2) of the MNN paper) and the 1x1 convolution
// (Section 3.3.2) are compute bound in fp32 long before they are memory bound.
// This kernel converts while it stages: every fp32 operand value x is split as
//     x = hi + lo + O(2^-17 |x|),   hi = bf16(x),  lo = bf16(x - hi)
// and the product is taken as hi*hi + hi*lo + lo*hi on the bf16 matrix cores
// (SPLIT = true, "bf16x3": about 16 mantissa bits per operand, three MFMAs
// instead of eight fp32 ones per 16 reduction rows), or as hi*hi alone
// (SPLIT = false: plain bf16 operands).  The tensors in memory stay fp32, so
// the transform kernels and the planner's layouts are shared with the fp32 path.
//
// Staging: a thread loads the same four columns of two consecutive reduction
// rows, rounds them to bf16 (RNE) and packs the row pair into one dword per
// column; LDS holds [row pair][column] dwords (hi and lo planes), written as
// 16-byte stores and read back conflict-free: an MFMA operand (lane l: rows
// 8*(l/32) .. +7, column l%32) is four dwords, row pairs 4*(l/32) .. +3.
#include <hip/hip_runtime.h>
#include "kernels.hpp"
#include "xcd_remap.hpp"
#include "gemm_epilogue.hpp"

namespace mnnconv {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

// round-to-nearest-even bf16 of x, as the upper 16 bits of a float pattern (inputs are finite)
__device__ __forceinline__ unsigned bf16_bits(float x)
{
    const unsigned u = __float_as_uint(x);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// packs rows (r, r+1) of one column: low half = row r.  *lo gets the packed residuals.
__device__ __forceinline__ void split_pair(float x0, float x1, unsigned* hi, unsigned* lo)
{
    const unsigned h0 = bf16_bits(x0), h1 = bf16_bits(x1);
    *hi = h0 | (h1 << 16);
    const float r0 = x0 - __uint_as_float(h0 << 16);
    const float r1 = x1 - __uint_as_float(h1 << 16);
    *lo = bf16_bits(r0) | (bf16_bits(r1) << 16);
}

// MODE 0: B element by element through (col / L, col % L); 1: 16-byte loads; 2: im2col gather.
template <int BM, int BN, int BK, int WM, int WN, int MODE, bool SPLIT>
__global__ __launch_bounds__(WM * WN * 64) void gemm_bf16_kernel(GemmProblem p, int tilesM, int tilesN, int total,
                                                                 int vecD, int ldc)
{
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32;
    constexpr int TN = BN / WN / 32;
    constexpr int RP = BK / 2;                // row pairs per chunk
    constexpr int A4 = RP * BM / 4;           // (row pair, 4 columns) slots of the A tile
    constexpr int B4 = RP * BN / 4;
    constexpr int LA = A4 / NT;
    constexpr int LB = B4 / NT;
    constexpr int NP = SPLIT ? 2 : 1;         // planes: hi (and lo)
    static_assert(A4 % NT == 0 && B4 % NT == 0, "tile must divide evenly over the workgroup");
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && BK % 16 == 0, "tile shape");

    // one LDS block: operand double buffer during the reduction, staging tiles for the result stores after it
    constexpr int AB_WORDS = 2 * NP * RP * (BM + BN);
    constexpr int C_WORDS = (NT / 64) * kStageFloats;
    __shared__ __attribute__((aligned(16))) unsigned smem[AB_WORDS > C_WORDS ? AB_WORDS : C_WORDS];
    unsigned (*As)[NP][RP][BM] = reinterpret_cast<unsigned (*)[NP][RP][BM]>(smem);
    unsigned (*Bs)[NP][RP][BN] = reinterpret_cast<unsigned (*)[NP][RP][BN]>(smem + 2 * NP * RP * BM);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;

    const int splitk = p.splitk > 1 ? p.splitk : 1;
    const int wg = (int)xcd_contiguous(blockIdx.x, (unsigned)(total * splitk));
    const int logical = wg / splitk;          // slices of one tile are neighbours: same XCD, same L2
    const int split = wg % splitk;
    const int tm = logical % tilesM;
    const int t2 = logical / tilesM;
    const int tn = t2 % tilesN;
    const int b = t2 / tilesN;
    const int m0 = tm * BM, n0 = tn * BN;

    const float* __restrict__ Ab = p.At + (long long)b * p.strideA_batch;
    const float* __restrict__ Bb = p.B + (long long)b * p.strideB_batch;

    int a_rp[LA], a_col[LA];
    bool a_ok[LA];
#pragma unroll
    for (int j = 0; j < LA; ++j) {
        const int s = tid + j * NT;
        a_rp[j] = s / (BM / 4);
        a_col[j] = (s % (BM / 4)) * 4;
        a_ok[j] = (m0 + a_col[j]) < p.lda;
    }
    constexpr bool VEC = (MODE == 1);
    int b_rp[LB], b_col[LB];
    long long b_off[LB][VEC ? 1 : 4];
    bool b_ok[LB][VEC ? 1 : 4];
    int g_y[LB][MODE == 2 ? 4 : 1], g_x[LB][MODE == 2 ? 4 : 1];
#pragma unroll
    for (int j = 0; j < LB; ++j) {
        const int s = tid + j * NT;
        b_rp[j] = s / (BN / 4);
        b_col[j] = (s % (BN / 4)) * 4;
#pragma unroll
        for (int e = 0; e < (VEC ? 1 : 4); ++e) {
            const int col = n0 + b_col[j] + e;
            b_ok[j][e] = col < p.Ncols;
            const int img = col / p.L, rest = col % p.L;
            if constexpr (MODE == 2) {
                b_off[j][e] = (long long)img * p.cv_C * p.cv_H * p.cv_W;
                g_y[j][e] = (rest / p.cv_Wo) * p.cv_sh - p.cv_ph;
                g_x[j][e] = (rest % p.cv_Wo) * p.cv_sw - p.cv_pw;
            } else {
                b_off[j][e] = (long long)img * p.strideB_img + rest;
            }
        }
    }

    // one row of B for slot j: four consecutive columns
    auto load_b_row = [&](int j, int r) -> float4 {
        const bool rok = r < p.R;
        if constexpr (MODE == 2) {
            const int taps = p.cv_kh * p.cv_kw;
            const int c = r / taps, rem = r % taps;
            const int dy = (rem / p.cv_kw) * p.cv_dh, dx = (rem % p.cv_kw) * p.cv_dw;
            const float* plane = Bb + (long long)c * p.cv_H * p.cv_W;
            float v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int iy = g_y[j][e] + dy, ix = g_x[j][e] + dx;
                const bool ok = rok && b_ok[j][e] && iy >= 0 && iy < p.cv_H && ix >= 0 && ix < p.cv_W;
                v[e] = ok ? plane[b_off[j][e] + (long long)iy * p.cv_W + ix] : 0.f;
            }
            return make_float4(v[0], v[1], v[2], v[3]);
        } else {
            const float* rowp = Bb + (long long)r * p.strideB_row;
            if constexpr (VEC) {
                if (rok && b_ok[j][0]) return *reinterpret_cast<const float4*>(rowp + b_off[j][0]);
                return make_float4(0.f, 0.f, 0.f, 0.f);
            } else {
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (rok && b_ok[j][e]) ? rowp[b_off[j][e]] : 0.f;
                return make_float4(v[0], v[1], v[2], v[3]);
            }
        }
    };

    float4 ra[LA][2], rb[LB][2];
    auto load_global = [&](int r0) {
#pragma unroll
        for (int j = 0; j < LA; ++j)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int r = r0 + 2 * a_rp[j] + h;
                if (a_ok[j] && r < p.R)
                    ra[j][h] = *reinterpret_cast<const float4*>(Ab + (long long)r * p.lda + m0 + a_col[j]);
                else
                    ra[j][h] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
        for (int j = 0; j < LB; ++j)
#pragma unroll
            for (int h = 0; h < 2; ++h) rb[j][h] = load_b_row(j, r0 + 2 * b_rp[j] + h);
    };
    auto pack = [&](const float4& x0, const float4& x1, uintx4* hi, uintx4* lo) {
        unsigned h[4], l[4];
        split_pair(x0.x, x1.x, &h[0], &l[0]);
        split_pair(x0.y, x1.y, &h[1], &l[1]);
        split_pair(x0.z, x1.z, &h[2], &l[2]);
        split_pair(x0.w, x1.w, &h[3], &l[3]);
        *hi = uintx4{h[0], h[1], h[2], h[3]};
        *lo = uintx4{l[0], l[1], l[2], l[3]};
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            uintx4 hi, lo;
            pack(ra[j][0], ra[j][1], &hi, &lo);
            *reinterpret_cast<uintx4*>(&As[buf][0][a_rp[j]][a_col[j]]) = hi;
            if constexpr (SPLIT) *reinterpret_cast<uintx4*>(&As[buf][NP - 1][a_rp[j]][a_col[j]]) = lo;
        }
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            uintx4 hi, lo;
            pack(rb[j][0], rb[j][1], &hi, &lo);
            *reinterpret_cast<uintx4*>(&Bs[buf][0][b_rp[j]][b_col[j]]) = hi;
            if constexpr (SPLIT) *reinterpret_cast<uintx4*>(&Bs[buf][NP - 1][b_rp[j]][b_col[j]]) = lo;
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int all_chunks = (p.R + BK - 1) / BK;
    const int per_split = (all_chunks + splitk - 1) / splitk;
    const int ch0 = split * per_split;
    const int nchunks = (all_chunks - ch0 < per_split ? all_chunks - ch0 : per_split);   // launcher guarantees >= 1
    load_global(ch0 * BK);
    store_lds(0);
    __syncthreads();

    const int lrow = lane >> 5;
    const int lcol = lane & 31;
    const int am = wm * (BM / WM) + lcol;
    const int bn = wn * (BN / WN) + lcol;

    auto operand = [&](const unsigned* plane_base, int ld, int ks, int col) -> bf16x8 {
        // row pairs 8*ks + 4*lrow + d, d = 0..3, of column col
        const unsigned* q = plane_base + (ks * 8 + lrow * 4) * ld + col;
        uintx4 v = uintx4{q[0], q[ld], q[2 * ld], q[3 * ld]};
        return __builtin_bit_cast(bf16x8, v);
    };

    for (int ch = 0; ch < nchunks; ++ch) {
        const int buf = ch & 1;
        if (ch + 1 < nchunks) load_global((ch0 + ch + 1) * BK);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 ah[TM], al[TM], bh[TN], bl[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                ah[i] = operand(&As[buf][0][0][0], BM, ks, am + i * 32);
                if constexpr (SPLIT) al[i] = operand(&As[buf][NP - 1][0][0], BM, ks, am + i * 32);
            }
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                bh[j] = operand(&Bs[buf][0][0][0], BN, ks, bn + j * 32);
                if constexpr (SPLIT) bl[j] = operand(&Bs[buf][NP - 1][0][0], BN, ks, bn + j * 32);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    if constexpr (SPLIT) {
                        // small terms first
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc[i][j], 0, 0, 0);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc[i][j], 0, 0, 0);
                    }
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], acc[i][j], 0, 0, 0);
                }
        }
        if (ch + 1 < nchunks) store_lds(buf ^ 1);
        __syncthreads();
    }

    const TileDest dest = tile_dest(p, b, split, splitk, ldc);
    store_tiles<TM, TN>(acc, dest, p.M, p.Ncols, m0 + wm * (BM / WM), n0 + wn * (BN / WN), lane,
                        reinterpret_cast<float*>(smem) + wave * kStageFloats, vecD);
}

template <int BM, int BN, int BK, int WM, int WN>
hipError_t launch_cfg(const GemmProblem& p, bool vec, hipStream_t s)
{
    const int tilesM = (p.M + BM - 1) / BM;
    const int tilesN = (p.Ncols + BN - 1) / BN;
    const long long total = (long long)tilesM * tilesN * p.batch;
    if (total <= 0 || total >= (1ll << 31)) return hipErrorInvalidValue;
    const int splitk = p.splitk > 1 ? p.splitk : 1;
    if (splitk > 1) {
        // every slice needs at least one chunk, and the scratch buffers must be there
        const int all_chunks = (p.R + BK - 1) / BK;
        const int per_split = (all_chunks + splitk - 1) / splitk;
        if ((long long)(splitk - 1) * per_split >= all_chunks || !p.splitk_partial || total * splitk >= (1ll << 31))
            return hipErrorInvalidValue;
    }
    const dim3 grid((unsigned)(total * splitk)), block(WM * WN * 64);
    const bool split = p.prec == 2;
    const int vecD = result_rows_vectorisable(p);
    const int ldc = gemm_splitk_ldc(p);
#define MNN_LAUNCH(MODE_)                                                                                         \
    do {                                                                                                          \
        if (split)                                                                                                \
            hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, BK, WM, WN, MODE_, true>), grid, block, 0, s, p, tilesM,  \
                               tilesN, (int)total, vecD, ldc);                                                    \
        else                                                                                                      \
            hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, BK, WM, WN, MODE_, false>), grid, block, 0, s, p, tilesM, \
                               tilesN, (int)total, vecD, ldc);                                                    \
    } while (0)
    if (p.gather) MNN_LAUNCH(2);
    else if (vec) MNN_LAUNCH(1);
    else MNN_LAUNCH(0);
#undef MNN_LAUNCH
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess || splitk == 1) return e;
    return launch_splitk_reduce(p, s);
}

inline bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

struct Variant { const char* name; hipError_t (*fn)(const GemmProblem&, bool, hipStream_t); int bm, bn, bk; };
const Variant kVariants[] = {
    {"auto", nullptr, 0, 0, 0},
    {"bf16_128x128x32_w2x2", launch_cfg<128, 128, 32, 2, 2>, 128, 128, 32},
    {"bf16_64x128x32_w1x4", launch_cfg<64, 128, 32, 1, 4>, 64, 128, 32},
    {"bf16_128x64x32_w2x2", launch_cfg<128, 64, 32, 2, 2>, 128, 64, 32},
    {"bf16_64x64x32_w2x2", launch_cfg<64, 64, 32, 2, 2>, 64, 64, 32},
    {"bf16_128x128x16_w2x2", launch_cfg<128, 128, 16, 2, 2>, 128, 128, 16},
    {"bf16_64x64x64_w2x2", launch_cfg<64, 64, 64, 2, 2>, 64, 64, 64},
    {"bf16_256x128x32_w4x2", launch_cfg<256, 128, 32, 4, 2>, 256, 128, 32},
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));

}  // namespace

bool gemm_bf16_variant_tile(int v, int* bm, int* bn, int* bk)
{
    if (v < 1 || v >= kNumVariants) return false;
    *bm = kVariants[v].bm; *bn = kVariants[v].bn; *bk = kVariants[v].bk;
    return true;
}

int gemm_bf16_variant_count() { return kNumVariants; }
const char* gemm_bf16_variant_name(int v) { return (v >= 0 && v < kNumVariants) ? kVariants[v].name : nullptr; }

hipError_t launch_gemm_bf16(const GemmProblem& p, hipStream_t s)
{
    if (!p.At || !p.B || !p.D) return hipErrorInvalidValue;
    if (p.M <= 0 || p.Ncols <= 0 || p.R <= 0 || p.batch <= 0 || p.L <= 0) return hipErrorInvalidValue;
    if (p.lda < p.M || (p.lda & 3) || !aligned16(p.At) || (p.strideA_batch & 3)) return hipErrorInvalidValue;
    if (p.prec != 1 && p.prec != 2) return hipErrorInvalidValue;
    if (p.variant < 0 || p.variant >= kNumVariants) return hipErrorInvalidValue;
    if (p.gather) {
        if (p.cv_C <= 0 || p.cv_H <= 0 || p.cv_W <= 0 || p.cv_kh <= 0 || p.cv_kw <= 0 || p.cv_sh <= 0 || p.cv_sw <= 0 ||
            p.cv_dh <= 0 || p.cv_dw <= 0 || p.cv_Wo <= 0 || p.L % p.cv_Wo != 0 || p.R != p.cv_C * p.cv_kh * p.cv_kw)
            return hipErrorInvalidValue;
    }
    const bool vec = aligned16(p.B) && (p.L % 4 == 0) && (p.Ncols % 4 == 0) && (p.strideB_batch % 4 == 0) &&
                     (p.strideB_img % 4 == 0) && (p.strideB_row % 4 == 0);
    int v = p.variant;
    if (v == 0) v = (p.M <= 64) ? 2 : 1;
    return kVariants[v].fn(p, vec, s);
}

}  // namespace mnnconv
