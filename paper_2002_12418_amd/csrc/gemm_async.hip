// Batched fp32 GEMM for gfx950, persistent and fully asynchronous.
//
//   D_b[m][col] = sum_r At_b[r][m] * B_b[r][col] (+ bias[m])
//
// the "basic matrix multiplication" unit (Sections 3.3.1 (2), 3.3.2 and 3.5 of
// the MNN paper) behind the Winograd-domain products and the 1x1 convolution.
//
// What is specific to this machine:
//  * Workgroups are persistent.  Each one walks a list of output tiles and the
//    operand stream never stops at a tile boundary: while the accumulators of
//    tile i are written out, the first chunks of tile i+1 are already landing.
//    Short reductions (R = C = 64..128 for the early layers) would otherwise
//    spend most of their time in the fill and drain of every tile.
//  * Operands go global memory -> LDS directly (buffer_load_dwordx4 ... lds),
//    1 KiB per wavefront-wide instruction, into a ring of NS stages.  The
//    buffer descriptor's range check zero-fills everything outside the matrix,
//    so ragged tiles need no separate code.
//  * One extra wavefront per workgroup does nothing but issue these copies and
//    wait for them (vmcnt); the WM x WN compute wavefronts only read LDS, issue
//    v_mfma_f32_32x32x2_f32 and store results.  Their stores therefore never
//    sit in the same counter as the prefetches, and one s_barrier per chunk is
//    the only synchronisation.
//  * The tile list is XCD-aware: the workgroups one XCD receives cover a
//    contiguous range of tiles at any moment (tiles along M fastest), so tiles
//    that share a B panel or an A batch meet in the same L2.
#include <hip/hip_runtime.h>
#include "kernels.hpp"

namespace mnnconv {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef int int32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) float lds_float;

constexpr int kXcds = 8;
constexpr unsigned kOob = 0x80000000u;        // byte offset beyond any descriptor range: reads give 0

__device__ __forceinline__ int xcd_remap(int v, int total)
{
    const int per = total / kXcds, rem = total % kXcds;
    const int xcd = v % kXcds, loc = v / kXcds;
    return xcd < rem ? xcd * (per + 1) + loc : rem * (per + 1) + (xcd - rem) * per + loc;
}

// Raw buffer descriptor over [base, base + bytes): stride 0, 32-bit elements, range checked.
__device__ __forceinline__ int32x4 make_rsrc(const void* base, unsigned bytes)
{
    const unsigned long long a = (unsigned long long)base;
    int32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)(a & 0xffffffffu));
    r[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((a >> 32) & 0xffffu));
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}

// 64 lanes x 16 bytes from the buffer to LDS[lds_addr + 16*lane ...]; lanes whose offset is out of
// range write zeros.  The compiler does not see this as an LDS write it has to order against; the
// caller waits on vmcnt and a barrier before anyone reads the stage.
__device__ __forceinline__ void copy_to_lds_16(int32x4 rsrc, unsigned lds_addr, unsigned voffset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voffset), "s"(rsrc)
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N <= 63, "vmcnt range");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

struct TileCoord { int b, m0, n0; };

template <int BM, int BN>
__device__ __forceinline__ TileCoord tile_coord(int v, int total, int tilesM, int tilesN)
{
    const int logical = xcd_remap(v, total);
    TileCoord t;
    const int tm = logical % tilesM;
    const int t2 = logical / tilesM;
    t.m0 = tm * BM;
    t.n0 = (t2 % tilesN) * BN;
    t.b = t2 / tilesN;
    return t;
}

template <int BM, int BN, int BK, int WM, int WN, int NS>
__global__ __launch_bounds__((WM * WN + 1) * 64) void gemm_f32_async_kernel(GemmProblem p, int tilesM, int tilesN,
                                                                           int total, unsigned a_bytes,
                                                                           unsigned b_bytes)
{
    constexpr int NW = WM * WN;               // compute wavefronts; wavefront NW is the copy wavefront
    constexpr int TM = BM / WM / 32;
    constexpr int TN = BN / WN / 32;
    constexpr int AQ = BK * BM / 256;         // 1 KiB copies per stage
    constexpr int BQ = BK * BN / 256;
    constexpr int LQ = AQ + BQ;
    static_assert((BK * BM) % 256 == 0 && (BK * BN) % 256 == 0, "stage must be whole KiB copies");
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && BK % 2 == 0, "tile shape");
    static_assert(NS >= 3 && (NS - 2) * LQ <= 63, "ring depth");

    __shared__ __attribute__((aligned(16))) float As[NS * BK * BM];
    __shared__ __attribute__((aligned(16))) float Bs[NS * BK * BN];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int G = gridDim.x;
    const int w = blockIdx.x;
    const int my_tiles = (total - w + G - 1) / G;          // tiles w, w + G, ...
    const int nchunks = (p.R + BK - 1) / BK;
    const int S = my_tiles * nchunks;                      // steps of this workgroup

    if (wave == NW) {
        // ------------------------------------------------------------ copy wavefront
        const unsigned as_base = (unsigned)(size_t)(lds_float*)As;
        const unsigned bs_base = (unsigned)(size_t)(lds_float*)Bs;
        // element this lane moves in copy j of a stage image [BK][BM] / [BK][BN]
        int a_row[AQ], a_col[AQ], b_row[BQ], b_col[BQ];
#pragma unroll
        for (int j = 0; j < AQ; ++j) { const int f = j * 256 + lane * 4; a_row[j] = f / BM; a_col[j] = f % BM; }
#pragma unroll
        for (int j = 0; j < BQ; ++j) { const int f = j * 256 + lane * 4; b_row[j] = f / BN; b_col[j] = f % BN; }

        int pt = 0, pch = 0;                                // producer cursor: tile index in my list, chunk
        unsigned a_off[AQ], b_off[BQ];                      // byte offsets at chunk 0, kOob if the column is outside
        int32x4 a_rsrc, b_rsrc;
        auto enter_tile = [&](int ti) {
            const TileCoord tc = tile_coord<BM, BN>(w + ti * G, total, tilesM, tilesN);
            a_rsrc = make_rsrc(p.At + (long long)tc.b * p.strideA_batch, a_bytes);
            b_rsrc = make_rsrc(p.B + (long long)tc.b * p.strideB_batch, b_bytes);
#pragma unroll
            for (int j = 0; j < AQ; ++j) {
                const int m = tc.m0 + a_col[j];
                a_off[j] = (m < p.lda) ? (unsigned)(a_row[j] * p.lda + m) * 4u : kOob;
            }
#pragma unroll
            for (int j = 0; j < BQ; ++j) {
                const int col = tc.n0 + b_col[j];
                const long long o = (long long)(col / p.L) * p.strideB_img + (col % p.L) + (long long)b_row[j] * p.strideB_row;
                b_off[j] = (col < p.Ncols) ? (unsigned)o * 4u : kOob;
            }
        };
        auto issue = [&](int st) {
            const int r0 = pch * BK;
            const unsigned a_add = (unsigned)(r0 * p.lda) * 4u;
            const unsigned b_add = (unsigned)((long long)r0 * p.strideB_row) * 4u;
#pragma unroll
            for (int j = 0; j < AQ; ++j) {
                const bool ok = (a_off[j] != kOob) && (r0 + a_row[j] < p.R);
                copy_to_lds_16(a_rsrc, as_base + (unsigned)((st * BK * BM + j * 256) * 4), ok ? a_off[j] + a_add : kOob);
            }
#pragma unroll
            for (int j = 0; j < BQ; ++j) {
                const bool ok = (b_off[j] != kOob) && (r0 + b_row[j] < p.R);
                copy_to_lds_16(b_rsrc, bs_base + (unsigned)((st * BK * BN + j * 256) * 4), ok ? b_off[j] + b_add : kOob);
            }
            if (++pch == nchunks) { pch = 0; ++pt; if (pt < my_tiles) enter_tile(pt); }
        };

        if (my_tiles > 0) enter_tile(0);
        int issued = 0;
#pragma unroll 1
        for (; issued < NS - 1 && issued < S; ++issued) issue(issued % NS);
        if (issued >= NS - 1) wait_vmcnt<(NS - 2) * LQ>(); else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();
#pragma unroll 1
        for (int s = 0; s < S; ++s) {
            // stage (s - 1) % NS was released by the barrier that ended step s - 1
            bool more = false;
            if (issued < S) { issue(issued % NS); ++issued; more = true; }
            // step s + 1 must have landed; the NS - 2 younger stages may stay in flight
            if (more) wait_vmcnt<(NS - 2) * LQ>(); else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
        }
        return;
    }

    // ---------------------------------------------------------------- compute wavefronts
    const int wm = wave % WM, wn = wave / WM;
    const int lrow = lane >> 5;               // which of the 2 reduction rows of an MFMA step
    const int lcol = lane & 31;
    const int am = wm * (BM / WM) + lcol;
    const int bn = wn * (BN / WN) + lcol;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    __builtin_amdgcn_s_barrier();             // stage 0 has landed
    asm volatile("" ::: "memory");            // LDS is written behind the compiler's back: no caching across barriers
    int s = 0;
#pragma unroll 1
    for (int ti = 0; ti < my_tiles; ++ti) {
#pragma unroll 1
        for (int ch = 0; ch < nchunks; ++ch, ++s) {
            const float* as = As + (s % NS) * (BK * BM);
            const float* bs = Bs + (s % NS) * (BK * BN);
#pragma unroll
            for (int kk = 0; kk < BK; kk += 2) {
                float av[TM], bv[TN];
#pragma unroll
                for (int i = 0; i < TM; ++i) av[i] = as[(kk + lrow) * BM + am + i * 32];
#pragma unroll
                for (int j = 0; j < TN; ++j) bv[j] = bs[(kk + lrow) * BN + bn + j * 32];
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
            }
            if (ch == nchunks - 1) {
                // ---- tile finished: lane holds column lcol of each 32x32 block, rows 8*(r/4) + 4*(lane/32) + r%4
                const TileCoord tc = tile_coord<BM, BN>(w + ti * G, total, tilesM, tilesN);
                float* __restrict__ Db = p.D + (long long)tc.b * p.strideD_batch;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int col = tc.n0 + wn * (BN / WN) + j * 32 + lcol;
                    const bool colok = col < p.Ncols;
                    const long long coff = (long long)(col / p.L) * p.strideD_img + (col % p.L);
#pragma unroll
                    for (int i = 0; i < TM; ++i) {
                        const int mbase = tc.m0 + wm * (BM / WM) + i * 32 + 4 * lrow;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int m = mbase + 8 * (r / 4) + (r % 4);
                            if (colok && m < p.M) {
                                float v = acc[i][j][r];
                                if (p.bias) v += p.bias[m];
                                Db[coff + (long long)m * p.strideD_row] = v;
                            }
                            acc[i][j][r] = 0.f;
                        }
                    }
                }
            }
            __builtin_amdgcn_s_barrier();     // everyone is done with this stage; the next one has landed
            asm volatile("" ::: "memory");
        }
    }
}

template <int BM, int BN, int BK, int WM, int WN, int NS>
hipError_t launch_async(const GemmProblem& p, hipStream_t s)
{
    const int tilesM = (p.M + BM - 1) / BM;
    const int tilesN = (p.Ncols + BN - 1) / BN;
    const long long total = (long long)tilesM * tilesN * p.batch;
    if (total <= 0 || total >= (1ll << 30)) return hipErrorInvalidValue;
    // extents of one batch of each operand, for the range-checked descriptors (offsets are 32-bit)
    const long long a_bytes = (long long)p.R * p.lda * 4;
    const long long imgs = (p.Ncols + p.L - 1) / p.L;
    const long long b_bytes = ((imgs - 1) * p.strideB_img + (long long)(p.R - 1) * p.strideB_row + p.L) * 4;
    if (a_bytes >= (1ll << 31) || b_bytes >= (1ll << 31) || a_bytes <= 0 || b_bytes <= 0) return hipErrorInvalidValue;
    // persistent grid: two workgroups per CU, a multiple of the XCD count unless there are fewer tiles
    int grid = 512;
    if (total < grid) grid = (int)total;
    if (grid >= kXcds) grid -= grid % kXcds;
    hipLaunchKernelGGL((gemm_f32_async_kernel<BM, BN, BK, WM, WN, NS>), dim3((unsigned)grid), dim3((WM * WN + 1) * 64), 0,
                       s, p, tilesM, tilesN, (int)total, (unsigned)a_bytes, (unsigned)b_bytes);
    return hipGetLastError();
}

inline bool aligned16(const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

struct AsyncVariant { const char* name; hipError_t (*fn)(const GemmProblem&, hipStream_t); int bm, bn; };
const AsyncVariant kAsync[] = {
    {"async_128x128x16_w2x2_s4", launch_async<128, 128, 16, 2, 2, 4>, 128, 128},
    {"async_64x128x16_w1x4_s4", launch_async<64, 128, 16, 1, 4, 4>, 64, 128},
    {"async_64x64x16_w2x2_s4", launch_async<64, 64, 16, 2, 2, 4>, 64, 64},
    {"async_128x64x16_w2x2_s4", launch_async<128, 64, 16, 2, 2, 4>, 128, 64},
    {"async_128x128x8_w2x2_s6", launch_async<128, 128, 8, 2, 2, 6>, 128, 128},
    {"async_256x128x16_w4x2_s3", launch_async<256, 128, 16, 4, 2, 3>, 256, 128},
    {"async_64x256x16_w1x4_s3", launch_async<64, 256, 16, 1, 4, 3>, 64, 256},
};
constexpr int kNumAsync = (int)(sizeof(kAsync) / sizeof(kAsync[0]));

}  // namespace

int gemm_f32_async_variant_count() { return kNumAsync; }
const char* gemm_f32_async_variant_name(int v) { return (v >= 0 && v < kNumAsync) ? kAsync[v].name : nullptr; }

// The direct-to-LDS path needs 16-byte granules on both operands: every run of 4 consecutive columns must be
// contiguous and aligned in memory.
bool gemm_f32_async_usable(const GemmProblem& p)
{
    if (!p.At || !p.B || !p.D) return false;
    if (p.M <= 0 || p.Ncols <= 0 || p.R <= 0 || p.batch <= 0 || p.L <= 0) return false;
    if (p.lda < p.M || (p.lda & 3) || !aligned16(p.At) || (p.strideA_batch & 3)) return false;
    return aligned16(p.B) && (p.L % 4 == 0) && (p.strideB_batch % 4 == 0) && (p.strideB_img % 4 == 0) &&
           (p.strideB_row % 4 == 0);
}

hipError_t launch_gemm_f32_async(const GemmProblem& p, int variant, hipStream_t s)
{
    if (!gemm_f32_async_usable(p)) return hipErrorInvalidValue;
    if (variant < 0 || variant >= kNumAsync) return hipErrorInvalidValue;
    return kAsync[variant].fn(p, s);
}

}  // namespace mnnconv
