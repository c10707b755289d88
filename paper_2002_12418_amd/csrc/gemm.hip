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
#include "xcd_remap.hpp"
#include "gemm_epilogue.hpp"

namespace mnnconv {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

// MODE 0: B read element by element through the (col / L, col % L) mapping; 1: the same with 16-byte
// loads; 2: B gathered from an NCHW tensor (implicit GEMM of the sliding-window convolution).
// PF: how many chunks ahead of the one being multiplied the global loads run (register stages).  One is
// enough when several workgroups share a CU; short grids (batch-1 layers) are bound by memory latency per
// chunk and want their whole slice of the reduction in flight at once.
//
// BUF: operands are read through buffer descriptors with 32-bit byte offsets; the hardware range check
// returns zero for an offset outside the operand, so ragged edges cost neither a branch nor a select and
// the compiler can count exactly how many loads are in flight (a branch around a load forces it to wait
// for all of them).  Needs every operand of one batch to span less than 2 GiB; larger ones take the
// pointer-based loader (BUF = false).
//
// WK: wavefronts along the reduction.  The WM x WN grid of wavefronts is repeated WK times; copy wk multiplies
// rows [wk * BK/WK, (wk+1) * BK/WK) of every chunk, and the WK partial blocks are added through LDS (in wk
// order) before the store.  A 32 x 32 output tile is one MFMA tile: with WK = 4 its reduction still runs on all
// four SIMDs of a CU, so that a problem with few output elements and a long reduction (batch-1 layers) spreads
// over four times as many workgroups without a second kernel.
template <int BM, int BN, int BK, int WM, int WN, int MODE, int PF = 1, bool BUF = true, int WK = 1>
__global__ __launch_bounds__(WM * WN * WK * 64) void gemm_f32_kernel(GemmProblem p, int tilesM, int tilesN, int total,
                                                                unsigned a_bytes, unsigned b_bytes, int vecD, int ldc)
{
    static_assert(PF == 1 || PF % 2 == 0, "the LDS buffer index is derived from the stage index");
    constexpr int NT = WM * WN * WK * 64;
    constexpr int KW = BK / WK;               // reduction rows of a chunk per wavefront
    constexpr int TM = BM / WM / 32;          // 32x32 tiles per wavefront along m
    constexpr int TN = BN / WN / 32;          // ... along columns
    constexpr int A4 = BK * BM / 4;           // float4 slots of the A tile
    constexpr int B4 = BK * BN / 4;
    constexpr int LA = A4 / NT;               // slots per thread
    constexpr int LB = B4 / NT;
    static_assert(A4 % NT == 0 && B4 % NT == 0, "tile must divide evenly over the workgroup");
    static_assert(BM % (WM * 32) == 0 && BN % (WN * 32) == 0 && BK % (2 * WK) == 0, "tile shape");

    // one LDS block: the operand double buffer during the reduction, per-wavefront 32x32 staging tiles
    // (row stride CS) for the vectorised result stores afterwards
    constexpr int AB_FLOATS = 2 * BK * (BM + BN);
    // and, behind those, the partial blocks of the wavefront copies wk > 0
    constexpr int C_FLOATS = WM * WN * kStageFloats;
    constexpr int RED_FLOATS = (WK - 1) * WM * WN * TM * TN * 16 * 64;
    __shared__ __attribute__((aligned(16))) float smem[AB_FLOATS > C_FLOATS + RED_FLOATS ? AB_FLOATS : C_FLOATS + RED_FLOATS];
    float (*As)[BK][BM] = reinterpret_cast<float (*)[BK][BM]>(smem);
    float (*Bs)[BK][BN] = reinterpret_cast<float (*)[BK][BN]>(smem + 2 * BK * BM);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wmn = wave % (WM * WN), wk = wave / (WM * WN);
    const int wm = wmn % WM, wn = wmn / WM;

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

    // ---- per-thread load slots (fixed over the K loop except for the row)
    constexpr bool VEC = (MODE == 1);
    constexpr int NE = VEC ? 1 : 4;           // loads per B slot
    constexpr unsigned kOutside = 0x80000000u;   // offset no operand reaches (all are < 2 GiB): reads as zero
    int a_row[LA], a_col[LA];
    int b_row[LB], b_col[LB];
#pragma unroll
    for (int j = 0; j < LA; ++j) {
        const int s = tid + j * NT;
        a_row[j] = s / (BM / 4);
        a_col[j] = (s % (BM / 4)) * 4;
    }
#pragma unroll
    for (int j = 0; j < LB; ++j) {
        const int s = tid + j * NT;
        b_row[j] = s / (BN / 4);
        b_col[j] = (s % (BN / 4)) * 4;
    }
    // gather (MODE 2): reduction row r = (c * kh + dy) * kw + dx is kept per slot as (c, dy, dx) and advanced
    // by BK rows per chunk without dividing; columns keep their image offset and top-left input coordinate
    int g_c[LB], g_dy[LB], g_dx[LB];
    int step_c = 0, step_dy = 0, step_dx = 0;
    int g_off[LB][MODE == 2 ? 4 : 1], g_y[LB][MODE == 2 ? 4 : 1], g_x[LB][MODE == 2 ? 4 : 1];
    bool b_ok[LB][NE];
    if constexpr (MODE == 2) {
#pragma unroll
        for (int j = 0; j < LB; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int col = n0 + b_col[j] + e;
                b_ok[j][e] = col < p.Ncols;
                const int img = col / p.L, rest = col % p.L;
                g_off[j][e] = img * p.cv_C * p.cv_H * p.cv_W;      // the launcher checked: fewer than 2^31 elements
                g_y[j][e] = (rest / p.cv_Wo) * p.cv_sh - p.cv_ph;
                g_x[j][e] = (rest % p.cv_Wo) * p.cv_sw - p.cv_pw;
            }
    }
    auto gather_advance = [&](int j) {
        g_c[j] += step_c;
        g_dy[j] += step_dy;
        g_dx[j] += step_dx;
        if (g_dx[j] >= p.cv_kw) { g_dx[j] -= p.cv_kw; g_dy[j] += 1; }
        if (g_dy[j] >= p.cv_kh) { g_dy[j] -= p.cv_kh; g_c[j] += 1; }
    };

    float4 ra[PF][LA], rb[PF][LB];

    // -- loader through buffer descriptors
    unsigned a_base[LA], b_base[LB][NE];       // byte offset of the slot in row 0, or kOutside
    __amdgpu_buffer_rsrc_t rsA, rsB;
    if constexpr (BUF) {
        rsA = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(Ab), 0, (int)a_bytes, 0x00020000);
        rsB = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(Bb), 0, (int)b_bytes, 0x00020000);
#pragma unroll
        for (int j = 0; j < LA; ++j)
            a_base[j] = (m0 + a_col[j]) < p.lda ? (unsigned)(m0 + a_col[j]) * 4u : kOutside;
        if constexpr (MODE != 2) {
#pragma unroll
            for (int j = 0; j < LB; ++j)
#pragma unroll
                for (int e = 0; e < NE; ++e) {
                    const int col = n0 + b_col[j] + e;
                    const int img = col / p.L, rest = col % p.L;
                    b_base[j][e] = col < p.Ncols ? (unsigned)(img * (int)p.strideB_img + rest) * 4u : kOutside;
                }
        }
    }
    auto load_buf = [&](int st, int r0) {
        // A: rows past R lie behind the end of the descriptor and read as zero by themselves
#pragma unroll
        for (int j = 0; j < LA; ++j) {
            const unsigned off = a_base[j] + (unsigned)(r0 + a_row[j]) * (unsigned)p.lda * 4u;
            const uint4v v = __builtin_amdgcn_raw_buffer_load_b128(rsA, (int)off, 0, 0);
            ra[st][j] = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
        }
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            if constexpr (MODE == 2) {
                const int c = g_c[j];
                const int dy = g_dy[j] * p.cv_dh, dx = g_dx[j] * p.cv_dw;
                const bool cok = c < p.cv_C;                       // same as r < R
                const int coff = c * p.cv_H * p.cv_W;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int iy = g_y[j][e] + dy, ix = g_x[j][e] + dx;
                    const bool ok = cok && b_ok[j][e] && (unsigned)iy < (unsigned)p.cv_H && (unsigned)ix < (unsigned)p.cv_W;
                    const unsigned off = ok ? (unsigned)(g_off[j][e] + coff + iy * p.cv_W + ix) * 4u : kOutside;
                    v[e] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsB, (int)off, 0, 0));
                }
                rb[st][j] = make_float4(v[0], v[1], v[2], v[3]);
                gather_advance(j);
            } else {
                // B: a row past R may lie inside the operand (next image / next plane), so it is masked
                const int r = r0 + b_row[j];
                const unsigned roff = r < p.R ? (unsigned)r * (unsigned)p.strideB_row * 4u : kOutside;
                if constexpr (VEC) {
                    const uint4v v = __builtin_amdgcn_raw_buffer_load_b128(rsB, (int)(b_base[j][0] | roff) < 0 ? (int)kOutside : (int)(b_base[j][0] + roff), 0, 0);
                    rb[st][j] = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
                } else {
                    float v[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const unsigned off = (int)(b_base[j][e] | roff) < 0 ? kOutside : b_base[j][e] + roff;
                        v[e] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rsB, (int)off, 0, 0));
                    }
                    rb[st][j] = make_float4(v[0], v[1], v[2], v[3]);
                }
            }
        }
    };

    // -- loader through 64-bit addresses (operands of 2 GiB and more)
    bool a_ok[LA];
    long long b_off[LB][NE];
    if constexpr (!BUF) {
#pragma unroll
        for (int j = 0; j < LA; ++j) a_ok[j] = (m0 + a_col[j]) < p.lda;
        if constexpr (MODE != 2) {
#pragma unroll
            for (int j = 0; j < LB; ++j)
#pragma unroll
                for (int e = 0; e < NE; ++e) {
                    const int col = n0 + b_col[j] + e;
                    b_ok[j][e] = col < p.Ncols;
                    b_off[j][e] = (long long)(col / p.L) * p.strideB_img + col % p.L;
                }
        }
    }
    auto load_ptr = [&](int st, int r0) {
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
                const int c = g_c[j];
                const int dy = g_dy[j] * p.cv_dh, dx = g_dx[j] * p.cv_dw;
                const float* plane = Bb + (long long)c * p.cv_H * p.cv_W;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int iy = g_y[j][e] + dy, ix = g_x[j][e] + dx;
                    const bool ok = rok && b_ok[j][e] && (unsigned)iy < (unsigned)p.cv_H && (unsigned)ix < (unsigned)p.cv_W;
                    v[e] = ok ? plane[(long long)g_off[j][e] + (long long)iy * p.cv_W + ix] : 0.f;
                }
                rb[st][j] = make_float4(v[0], v[1], v[2], v[3]);
                gather_advance(j);
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
    auto load_global = [&](int st, int r0) {
        if constexpr (BUF) load_buf(st, r0);
        else load_ptr(st, r0);
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
    if constexpr (MODE == 2) {
        const int taps = p.cv_kh * p.cv_kw;
        step_c = BK / taps;
        step_dy = (BK % taps) / p.cv_kw;
        step_dx = (BK % taps) % p.cv_kw;
#pragma unroll
        for (int j = 0; j < LB; ++j) {
            const int r = ch0 * BK + b_row[j];
            const int rem = r % taps;
            g_c[j] = r / taps;
            g_dy[j] = rem / p.cv_kw;
            g_dx[j] = rem % p.cv_kw;
        }
    }
    // register stage u holds chunk c (c % PF == u) until it has been copied to LDS buffer c % 2;
    // load_global is called once per chunk, in chunk order (the gather state advances with each call)
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
            // operands of step kk + 2 are read from LDS while the MFMAs of step kk run
            float av[2][TM], bv[2][TN];
            const int k0 = wk * KW + lrow;    // this wavefront's rows of the chunk
#pragma unroll
            for (int i = 0; i < TM; ++i) av[0][i] = As[buf][k0][am + i * 32];
#pragma unroll
            for (int j = 0; j < TN; ++j) bv[0][j] = Bs[buf][k0][bn + j * 32];
#pragma unroll
            for (int kk = 0; kk < KW; kk += 2) {
                const int cur = (kk >> 1) & 1, nxt = cur ^ 1;
                if (kk + 2 < KW) {
#pragma unroll
                    for (int i = 0; i < TM; ++i) av[nxt][i] = As[buf][k0 + kk + 2][am + i * 32];
#pragma unroll
                    for (int j = 0; j < TN; ++j) bv[nxt][j] = Bs[buf][k0 + kk + 2][bn + j * 32];
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][i], bv[cur][j], acc[i][j], 0, 0, 0);
            }
            if (c + 1 < nchunks) store_lds(buf ^ 1, (u + 1) % PF);
            __syncthreads();
        }
    }

    // ---- the wavefront copies along the reduction add their blocks into copy 0 (fixed order: same bits every run)
    if constexpr (WK > 1) {
        float* red = smem + C_FLOATS;         // [wk - 1][wmn][tile][register][lane]; the operands are dead (barrier above)
        if (wk > 0) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        red[((((wk - 1) * (WM * WN) + wmn) * (TM * TN) + i * TN + j) * 16 + r) * 64 + lane] = acc[i][j][r];
        }
        __syncthreads();
        if (wk > 0) return;
#pragma unroll
        for (int w = 1; w < WK; ++w)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        acc[i][j][r] += red[((((w - 1) * (WM * WN) + wmn) * (TM * TN) + i * TN + j) * 16 + r) * 64 + lane];
    }

    // ---- results (or this slice's partial results) to memory
    const TileDest dest = tile_dest(p, b, split, splitk, ldc);
    store_tiles<TM, TN>(acc, dest, p.M, p.Ncols, m0 + wm * (BM / WM), n0 + wn * (BN / WN), lane,
                        smem + wmn * kStageFloats, vecD);
}

// Adds the split-K slices P[split][batch][M][ldc] in slice order, applies the bias and writes D.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmProblem p, int ldc, int vecD)
{
    const int q = ldc >> 2;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long rows = (long long)p.batch * p.M;
    if (idx >= rows * q) return;
    const int c4 = (int)(idx % q) * 4;
    const long long bm = idx / q;
    const int m = (int)(bm % p.M), b = (int)(bm / p.M);
    const float* src = p.splitk_partial + bm * ldc + c4;
    const long long slice = rows * ldc;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    int sl = 0;
    for (; sl + 4 <= p.splitk; sl += 4) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const float4*>(src + (long long)(sl + u) * slice);
#pragma unroll
        for (int u = 0; u < 4; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
    }
    for (; sl < p.splitk; ++sl) {
        const float4 v = *reinterpret_cast<const float4*>(src + (long long)sl * slice);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    if (p.bias) {
        const float bv = p.bias[m];
        s.x += bv; s.y += bv; s.z += bv; s.w += bv;
    }
    float* Db = p.D + (long long)b * p.strideD_batch + (long long)m * p.strideD_row;
    if (vecD) {
        *reinterpret_cast<float4*>(Db + (long long)(c4 / p.L) * p.strideD_img + (c4 % p.L)) = s;
    } else {
        const float o[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int col = c4 + e;
            if (col < p.Ncols) Db[(long long)(col / p.L) * p.strideD_img + (col % p.L)] = o[e];
        }
    }
}

// Bytes one batch of each operand spans, and whether the descriptor-based loader can address them.
struct Extents { unsigned a_bytes, b_bytes; bool narrow; };
Extents operand_extents(const GemmProblem& p)
{
    const long long a = (long long)p.R * p.lda * 4;
    long long b;
    const long long imgs = (p.Ncols + p.L - 1) / p.L;
    if (p.gather) b = imgs * p.cv_C * p.cv_H * p.cv_W * 4;
    else b = ((imgs - 1) * p.strideB_img + (long long)(p.R - 1) * p.strideB_row + p.L) * 4;
    Extents e;
    // offsets run a few chunks past the last row before the range check stops them: keep them below 2^31
    e.narrow = a > 0 && b > 0 && a < (1ll << 30) && b < (1ll << 31) - 64 && (long long)p.lda * 4 * 1024 < (1ll << 30) &&
               p.strideB_img >= 0 && p.strideB_row >= 0;
    e.a_bytes = e.narrow ? (unsigned)a : 0u;
    e.b_bytes = e.narrow ? (unsigned)b : 0u;
    return e;
}

template <int BM, int BN, int BK, int WM, int WN, int PF = 1, bool BUF = true, int WK = 1>
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
    const Extents ex = operand_extents(p);
    if (BUF && !ex.narrow) return hipErrorNotSupported;       // the caller falls back to the 64-bit loader
    const dim3 grid((unsigned)(total * splitk)), block(WM * WN * WK * 64);
    const int vecD = result_rows_vectorisable(p);
    const int ldc = gemm_splitk_ldc(p);
    if (p.gather)
        hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, BK, WM, WN, 2, PF, BUF, WK>), grid, block, 0, s, p, tilesM, tilesN,
                           (int)total, ex.a_bytes, ex.b_bytes, vecD, ldc);
    else if (vec)
        hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, BK, WM, WN, 1, PF, BUF, WK>), grid, block, 0, s, p, tilesM, tilesN,
                           (int)total, ex.a_bytes, ex.b_bytes, vecD, ldc);
    else
        hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, BK, WM, WN, 0, PF, BUF, WK>), grid, block, 0, s, p, tilesM, tilesN,
                           (int)total, ex.a_bytes, ex.b_bytes, vecD, ldc);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess || splitk == 1) return e;
    return launch_splitk_reduce(p, s);
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
    {"128x128x16_w4x2_pf2", launch_cfg<128, 128, 16, 4, 2, 2>, 128, 128, 16},
    {"128x128x16_w2x2_pf2", launch_cfg<128, 128, 16, 2, 2, 2>, 128, 128, 16},
    {"256x128x16_w4x2_pf2", launch_cfg<256, 128, 16, 4, 2, 2>, 256, 128, 16},
    {"128x128x32_w4x2_pf2", launch_cfg<128, 128, 32, 4, 2, 2>, 128, 128, 32},
    // small output tiles with the wavefronts of a workgroup spread along the reduction (k<WK>): four times the
    // workgroups of a 64 x 64 tile for outputs too small to fill the chip otherwise
    {"32x32x32_k4", launch_cfg<32, 32, 32, 1, 1, 1, true, 4>, 32, 32, 32},
    {"32x32x32_k4_pf2", launch_cfg<32, 32, 32, 1, 1, 2, true, 4>, 32, 32, 32},
    {"32x32x64_k4_pf2", launch_cfg<32, 32, 64, 1, 1, 2, true, 4>, 32, 32, 64},
    {"32x64x32_w1x2k2_pf2", launch_cfg<32, 64, 32, 1, 2, 2, true, 2>, 32, 64, 32},
    {"64x32x32_w2x1k2_pf2", launch_cfg<64, 32, 32, 2, 1, 2, true, 2>, 64, 32, 32},
};
constexpr int kNumVariants = (int)(sizeof(kVariants) / sizeof(kVariants[0]));
}  // namespace

// Variant ids: 0 = choose from the shape, 1 .. kNumVariants-1 = the tile configurations above.
int gemm_f32_variant_count() { return kNumVariants; }
const char* gemm_f32_variant_name(int v) { return (v >= 0 && v < kNumVariants) ? kVariants[v].name : nullptr; }

bool gemm_f32_variant_tile(int v, int* bm, int* bn, int* bk)
{
    if (v < 1 || v >= kNumVariants) return false;
    *bm = kVariants[v].bm; *bn = kVariants[v].bn; *bk = kVariants[v].bk;
    return true;
}

bool gemm_variant_tile(int prec, int variant, int* bm, int* bn, int* bk)
{
    return prec == 0 ? gemm_f32_variant_tile(variant, bm, bn, bk) : gemm_bf16_variant_tile(variant, bm, bn, bk);
}

long long gemm_splitk_workspace(const GemmProblem& p, int splitk)
{
    return (long long)splitk * p.batch * p.M * gemm_splitk_ldc(p);
}

hipError_t launch_splitk_reduce(const GemmProblem& p, hipStream_t s)
{
    if (p.splitk < 2 || !p.splitk_partial || !p.D) return hipErrorInvalidValue;
    const int ldc = gemm_splitk_ldc(p);
    const long long groups = (long long)p.batch * p.M * (ldc / 4);
    if (groups <= 0 || (groups + 255) / 256 >= (1ll << 31)) return hipErrorInvalidValue;
    GemmProblem q = p;
    q.splitk = 1;                                   // vectorisability of D itself, not of the scratch tensor
    const int vecD = result_rows_vectorisable(q);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, s, p, ldc, vecD);
    return hipGetLastError();
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
    }
    const bool vec = aligned16(p.B) && (p.L % 4 == 0) && (p.Ncols % 4 == 0) && (p.strideB_batch % 4 == 0) &&
                     (p.strideB_img % 4 == 0) && (p.strideB_row % 4 == 0);
    int v = p.variant;
    if (v == 0) v = (p.M <= 64) ? 2 : 1;
    const hipError_t e = kVariants[v].fn(p, vec, s);
    if (e != hipErrorNotSupported) return e;
    // an operand of 2 GiB or more per batch: one tile configuration with 64-bit addressing serves all variants
    if (p.splitk > 1) return hipErrorInvalidValue;              // split-K scratch was sized for another tile
    return launch_cfg<128, 128, 16, 2, 2, 1, false>(p, vec, s);
}

}  // namespace mnnconv
