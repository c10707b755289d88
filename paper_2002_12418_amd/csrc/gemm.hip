// Batched fp32 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x2_f32).
//
// This is the "basic matrix multiplication" unit everything compute-intensive
// is lowered to (Sections 3.3.1 (2) and 3.5 of the MNN paper): the alpha^2
// Winograd-domain products M_xi = U_xi V_xi and the 1x1 convolution
// y_n = w x_n + b.
//
//   D_b[m][col] = sum_r At_b[r][m] * B_b[r][col] (+ bias[m])
//
// Both operands are stored with the reduction index r as the slow dimension, so
// a [BK][BM] / [BK][BN] tile is a plain coalesced copy from global memory into
// LDS, and an MFMA operand (lane l holds element [r = l/32][m = l%32]) is one
// conflict-free ds_read_b32 per 32x32 tile.
//
// Workgroup: WM x WN wavefronts of 64 lanes; each wavefront owns a
// (BM/WM) x (BN/WN) block made of 32x32 MFMA tiles held in accumulator VGPRs.
// The K loop is double buffered through LDS with a register prefetch of the
// next chunk; one barrier per chunk.
//
// Grid: one-dimensional, remapped so that the workgroups one XCD receives
// (hardware deals consecutive workgroup ids round-robin to the 8 XCDs) are a
// contiguous range of tiles: tiles that share a B column panel and an A batch
// then hit the same L2.
#include <hip/hip_runtime.h>
#include "kernels.hpp"
#include "gemm_splitk.hpp"

namespace mnnconv {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kXcds = 8;

__device__ __forceinline__ int xcd_remap(int bid, int total)
{
    const int per = total / kXcds, rem = total % kXcds;
    const int xcd = bid % kXcds, loc = bid / kXcds;
    return xcd < rem ? xcd * (per + 1) + loc : rem * (per + 1) + (xcd - rem) * per + loc;
}

// MODE 0: B read element by element through the (col / L, col % L) mapping; 1: the same with 16-byte
// loads; 2: B gathered from an NCHW tensor (implicit GEMM of the sliding-window convolution).
// PF: how many chunks ahead of the one being multiplied the global loads run (register stages).  One is
// enough when several workgroups share a CU; short grids (batch-1 layers) are bound by memory latency per
// chunk and want their whole slice of the reduction in flight at once.
template <int BM, int BN, int BK, int WM, int WN, int MODE, int PF = 1>
__global__ __launch_bounds__(WM * WN * 64) void gemm_f32_kernel(GemmProblem p, int tilesM, int tilesN, int total)
{
    static_assert(PF == 1 || PF % 2 == 0, "the LDS buffer index is derived from the stage index");
    constexpr int NT = WM * WN * 64;
    constexpr int TM = BM / WM / 32;          // 32x32 tiles per wavefront along m
    constexpr int TN = BN / WN / 32;          // ... along columns
    constexpr int A4 = BK * BM / 4;           // float4 slots of the A tile
    constexpr int B4 = BK * BN / 4;
    constexpr int LA = A4 / NT;               // slots per thread
    constexpr int LB = B4 / NT;
    static_assert(A4 % NT == 0 && B4 % NT == 0, "tile must divide evenly over the workgroup");
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && BK % 2 == 0, "tile shape");

    __shared__ __attribute__((aligned(16))) float As[2][BK][BM];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK][BN];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;

    const int splitk = p.splitk > 1 ? p.splitk : 1;
    const int wg = xcd_remap((int)blockIdx.x, total * splitk);
    const int logical = wg / splitk;          // slices of one tile are neighbours: same XCD, same L2
    const int split = wg % splitk;
    const int tm = logical % tilesM;
    const int t2 = logical / tilesM;
    const int tn = t2 % tilesN;
    const int b = t2 / tilesN;
    const int m0 = tm * BM, n0 = tn * BN;

    const float* __restrict__ Ab = p.At + (long long)b * p.strideA_batch;
    const float* __restrict__ Bb = p.B + (long long)b * p.strideB_batch;

    // ---- per-thread load slots (fixed over the K loop except for the row)
    int a_row[LA], a_col[LA];
    bool a_ok[LA];
#pragma unroll
    for (int j = 0; j < LA; ++j) {
        const int s = tid + j * NT;
        a_row[j] = s / (BM / 4);
        a_col[j] = (s % (BM / 4)) * 4;
        a_ok[j] = (m0 + a_col[j]) < p.lda;
    }
    constexpr bool VEC = (MODE == 1);
    int b_row[LB], b_col[LB];
    long long b_off[LB][VEC ? 1 : 4];
    bool b_ok[LB][VEC ? 1 : 4];
    int g_y[LB][MODE == 2 ? 4 : 1], g_x[LB][MODE == 2 ? 4 : 1];   // gather: top-left input coordinate of the column
#pragma unroll
    for (int j = 0; j < LB; ++j) {
        const int s = tid + j * NT;
        b_row[j] = s / (BN / 4);
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

    float4 ra[PF][LA], rb[PF][LB];
    auto load_global = [&](int st, int r0) {
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            const int r = r0 + a_row[j];
            if (a_ok[j] && r < p.R)
                ra[st][j] = *reinterpret_cast<const float4*>(Ab + (long long)r * p.lda + m0 + a_col[j]);
            else
                ra[st][j] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            const int r = r0 + b_row[j];
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
                rb[st][j] = make_float4(v[0], v[1], v[2], v[3]);
                continue;
            }
            const float* rowp = Bb + (long long)r * p.strideB_row;
            if constexpr (VEC) {
                if (rok && b_ok[j][0])
                    rb[st][j] = *reinterpret_cast<const float4*>(rowp + b_off[j][0]);
                else
                    rb[st][j] = make_float4(0.f, 0.f, 0.f, 0.f);
            } else {
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (rok && b_ok[j][e]) ? rowp[b_off[j][e]] : 0.f;
                rb[st][j] = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
    };
    auto store_lds = [&](int buf, int st) {
#pragma unroll
        for (int j = 0; j < LA; ++j) *reinterpret_cast<float4*>(&As[buf][a_row[j]][a_col[j]]) = ra[st][j];
#pragma unroll
        for (int j = 0; j < LB; ++j) *reinterpret_cast<float4*>(&Bs[buf][b_row[j]][b_col[j]]) = rb[st][j];
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
    // register stage u holds chunk c (c % PF == u) until it has been copied to LDS buffer c % 2
#pragma unroll
    for (int u = 0; u < PF; ++u)
        if (u < nchunks) load_global(u, (ch0 + u) * BK);
    store_lds(0, 0);
    __syncthreads();

    const int lrow = lane >> 5;               // which of the 2 reduction rows of an MFMA step
    const int lcol = lane & 31;
    const int am = wm * (BM / WM) + lcol;
    const int bn = wn * (BN / WN) + lcol;

    for (int ch = 0; ch < nchunks; ch += PF) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int c = ch + u;
            if (c >= nchunks) break;
            const int buf = (PF == 1) ? (c & 1) : (u & 1);
            if (c + PF < nchunks) load_global(u, (ch0 + c + PF) * BK);
#pragma unroll
            for (int kk = 0; kk < BK; kk += 2) {
                float av[TM], bv[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) av[i] = As[buf][kk + lrow][am + i * 32];
#pragma unroll
                for (int j = 0; j < TN; ++j) bv[j] = Bs[buf][kk + lrow][bn + j * 32];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
            }
            if (c + 1 < nchunks) store_lds(buf ^ 1, (u + 1) % PF);
            __syncthreads();
        }
    }

    if (splitk > 1) {
        if (!splitk_combine<TM, TN, NT>(acc, p.splitk_partial, p.splitk_counters, logical, split, splitk, tid)) return;
    }
    // ---- epilogue: lane holds column lcol of each tile, rows 8*(r/4) + 4*(lane/32) + r%4
    float* __restrict__ Db = p.D + (long long)b * p.strideD_batch;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * (BN / WN) + j * 32 + lcol;
        if (col >= p.Ncols) continue;
        const long long coff = (long long)(col / p.L) * p.strideD_img + (col % p.L);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int mbase = m0 + wm * (BM / WM) + i * 32 + 4 * lrow;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = mbase + 8 * (r / 4) + (r % 4);
                if (m < p.M) {
                    float v = acc[i][j][r];
                    if (p.bias) v += p.bias[m];
                    Db[coff + (long long)m * p.strideD_row] = v;
                }
            }
        }
    }
}

template <int BM, int BN, int BK, int WM, int WN, int PF = 1>
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
        if ((long long)(splitk - 1) * per_split >= all_chunks || !p.splitk_partial || !p.splitk_counters || total * splitk >= (1ll << 31))
            return hipErrorInvalidValue;
    }
    if (p.gather)
        hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, BK, WM, WN, 2, PF>), dim3((unsigned)(total * splitk)), dim3(WM * WN * 64),
                           0, s, p, tilesM, tilesN, (int)total);
    else if (vec)
        hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, BK, WM, WN, 1, PF>), dim3((unsigned)(total * splitk)), dim3(WM * WN * 64),
                           0, s, p, tilesM, tilesN, (int)total);
    else
        hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, BK, WM, WN, 0, PF>), dim3((unsigned)(total * splitk)), dim3(WM * WN * 64),
                           0, s, p, tilesM, tilesN, (int)total);
    return hipGetLastError();
}

inline bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

}  // namespace

namespace {
struct Variant { const char* name; hipError_t (*fn)(const GemmProblem&, bool, hipStream_t); int bm, bn, bk; };
const Variant kVariants[] = {
    {"auto", nullptr, 0, 0, 0},
    {"128x128x16_w2x2", launch_cfg<128, 128, 16, 2, 2>, 128, 128, 16},
    {"64x128x16_w1x4", launch_cfg<64, 128, 16, 1, 4>, 64, 128, 16},
    {"128x128x32_w2x2", launch_cfg<128, 128, 32, 2, 2>, 128, 128, 32},
    {"128x64x16_w2x2", launch_cfg<128, 64, 16, 2, 2>, 128, 64, 16},
    {"128x64x32_w2x2", launch_cfg<128, 64, 32, 2, 2>, 128, 64, 32},
    {"256x128x16_w4x2", launch_cfg<256, 128, 16, 4, 2>, 256, 128, 16},
    {"64x64x16_w2x2", launch_cfg<64, 64, 16, 2, 2>, 64, 64, 16},
    {"64x64x32_w2x2", launch_cfg<64, 64, 32, 2, 2>, 64, 64, 32},
    {"128x128x16_w4x2", launch_cfg<128, 128, 16, 4, 2>, 128, 128, 16},
    {"64x128x32_w1x4", launch_cfg<64, 128, 32, 1, 4>, 64, 128, 32},
    {"64x256x16_w1x4", launch_cfg<64, 256, 16, 1, 4>, 64, 256, 16},
    // deeper global-load pipelines for grids too short to hide memory latency by occupancy
    {"64x64x32_w2x2_pf2", launch_cfg<64, 64, 32, 2, 2, 2>, 64, 64, 32},
    {"64x64x32_w2x2_pf4", launch_cfg<64, 64, 32, 2, 2, 4>, 64, 64, 32},
    {"64x64x16_w2x2_pf4", launch_cfg<64, 64, 16, 2, 2, 4>, 64, 64, 16},
    {"128x64x32_w2x2_pf2", launch_cfg<128, 64, 32, 2, 2, 2>, 128, 64, 32},
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));
}  // namespace

// Variant ids: 0 = choose from the shape, 1 .. kNumVariants-1 = register-staged tiles of this file,
// kNumVariants .. = the persistent direct-to-LDS kernels.
int gemm_f32_variant_count() { return kNumVariants + gemm_f32_async_variant_count(); }
const char* gemm_f32_variant_name(int v)
{
    if (v >= 0 && v < kNumVariants) return kVariants[v].name;
    return gemm_f32_async_variant_name(v - kNumVariants);
}

bool gemm_f32_variant_tile(int v, int* bm, int* bn, int* bk)
{
    if (v < 1 || v >= kNumVariants) return false;       // the persistent kernels do not split K
    *bm = kVariants[v].bm; *bn = kVariants[v].bn; *bk = kVariants[v].bk;
    return true;
}

bool gemm_variant_tile(int prec, int variant, int* bm, int* bn, int* bk)
{
    return prec == 0 ? gemm_f32_variant_tile(variant, bm, bn, bk) : gemm_bf16_variant_tile(variant, bm, bn, bk);
}

void gemm_splitk_workspace(const GemmProblem& p, int bm, int bn, int splitk, long long* partial_floats, long long* counters)
{
    const long long tiles = (long long)((p.M + bm - 1) / bm) * ((p.Ncols + bn - 1) / bn) * p.batch;
    *counters = tiles;
    *partial_floats = tiles * splitk * bm * bn;
}

hipError_t launch_gemm_f32(const GemmProblem& p, hipStream_t s)
{
    if (p.prec != 0) return launch_gemm_bf16(p, s);
    if (!p.At || !p.B || !p.D) return hipErrorInvalidValue;
    if (p.M <= 0 || p.Ncols <= 0 || p.R <= 0 || p.batch <= 0 || p.L <= 0) return hipErrorInvalidValue;
    if (p.lda < p.M || (p.lda & 3) || !aligned16(p.At) || (p.strideA_batch & 3)) return hipErrorInvalidValue;
    if (p.variant < 0 || p.variant >= gemm_f32_variant_count()) return hipErrorInvalidValue;
    if (p.gather) {
        if (p.cv_C <= 0 || p.cv_H <= 0 || p.cv_W <= 0 || p.cv_kh <= 0 || p.cv_kw <= 0 || p.cv_sh <= 0 || p.cv_sw <= 0 ||
            p.cv_dh <= 0 || p.cv_dw <= 0 || p.cv_Wo <= 0 || p.L % p.cv_Wo != 0 || p.R != p.cv_C * p.cv_kh * p.cv_kw)
            return hipErrorInvalidValue;
        if (p.variant >= kNumVariants) return hipErrorInvalidValue;   // the direct-to-LDS kernels cannot gather
    }
    if (p.variant >= kNumVariants) {
        if (p.splitk > 1) return hipErrorInvalidValue;
        return launch_gemm_f32_async(p, p.variant - kNumVariants, s);
    }
    const bool vec = aligned16(p.B) && (p.L % 4 == 0) && (p.Ncols % 4 == 0) && (p.strideB_batch % 4 == 0) &&
                     (p.strideB_img % 4 == 0) && (p.strideB_row % 4 == 0);
    int v = p.variant;
    if (v == 0) v = (p.M <= 64) ? 2 : 1;
    return kVariants[v].fn(p, vec, s);
}

}  // namespace mnnconv
