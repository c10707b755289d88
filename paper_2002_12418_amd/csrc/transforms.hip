// Winograd transform kernels for gfx950 (Section 3.3.1 of the MNN paper:
// Y = A^T [ sum_channel (G W G^T) (.) (B^T X B) ] A).
//
// All three are bandwidth bound (a few FLOP per byte moved), so the layout is
// chosen for coalescing: one lane owns one (channel, tile) pair, consecutive
// lanes own consecutive tiles, and every store / load of the Winograd-domain
// tensors V[xi][c][p] and M[xi][k][p] is contiguous across the wavefront.
// The transform matrices arrive as kernel arguments, so they sit in SGPRs and
// every multiply is a v_fma with a scalar operand.
#include <hip/hip_runtime.h>
#include <type_traits>
#include "kernels.hpp"
#include "xcd_remap.hpp"

namespace mnnconv {

namespace {

constexpr int kMaxK = 7;   // largest kernel size with a Winograd path

// ---------------------------------------------------------------- filter: U = G w G^T
struct FilterMat { float g[kMaxAlphaT][kMaxK]; };

// KT = taps per axis.  The rows of G are walked in loops that stay rolled (alpha is a run-time value) while every
// array index is a compile-time constant, so the kernel weights, one row of G w and nothing else live in registers.
template <int KT>
__global__ __launch_bounds__(256) void filter_transform_kernel(WinoGeom g, FilterMat gm,
                                                               const float* __restrict__ w,
                                                               float* __restrict__ U)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)g.K * g.C) return;
    const int kk = (int)(idx % g.K);
    const int c = (int)(idx / g.K);
    const int a = g.alpha;
    const float* wp = w + ((long long)kk * g.C + c) * KT * KT;
    float wl[KT][KT];
#pragma unroll
    for (int r = 0; r < KT; ++r)
#pragma unroll
        for (int s = 0; s < KT; ++s) wl[r][s] = wp[r * KT + s];
#pragma unroll 1
    for (int i = 0; i < a; ++i) {
        // row i of G w  (k values)
        float row[KT];
#pragma unroll
        for (int s = 0; s < KT; ++s) {
            float acc = 0.f;
#pragma unroll
            for (int r = 0; r < KT; ++r) acc = fmaf(gm.g[i][r], wl[r][s], acc);
            row[s] = acc;
        }
        // row i of U = (G w) G^T
#pragma unroll 1
        for (int j = 0; j < a; ++j) {
            float acc = 0.f;
#pragma unroll
            for (int s = 0; s < KT; ++s) acc = fmaf(row[s], gm.g[j][s], acc);
            if (g.blocked)   // Ub[b = j][c/4][a = i][k/16][c%4][k%16]
                U[(((((long long)j * g.cchunks + (c >> 2)) * a + i) * g.kg + (kk >> 4)) << 6) + ((c & 3) << 4) + (kk & 15)] = acc;
            else
                U[((long long)(i * a + j) * g.C + c) * g.ldk + kk] = acc;
        }
    }
}

// 16- and 8-byte loads at 4-byte alignment (global memory takes them at any dword alignment)
struct __attribute__((packed, aligned(4))) Unaligned4 { float x, y, z, w; };
struct __attribute__((packed, aligned(4))) Unaligned2 { float x, y; };

// ---------------------------------------------------------------- input: V = B^T d B
// Division of a value below 2^31 by a constant the host knows: q = mulhi(n, m) >> sh with m = ceil(2^(31+L) / d),
// L = ceil(log2 d), sh = L - 1 (exact for every n < 2^31).  A run-time division costs some thirty vector instructions,
// and this kernel's instruction count is part of its time.
struct FastDiv { unsigned m, sh, d; };
inline FastDiv make_fastdiv(unsigned d)
{
    FastDiv f{0u, 0u, d};
    if (d <= 1) return f;
    unsigned L = 0;
    while ((1u << L) < d) ++L;
    f.m = (unsigned)((((unsigned long long)1 << (31 + L)) + d - 1) / d);
    f.sh = L - 1;
    return f;
}
__device__ __forceinline__ unsigned fast_div(unsigned n, const FastDiv& f) { return f.d <= 1 ? n : (__umulhi(n, f.m) >> f.sh); }

struct InputMap { FastDiv by_tw, by_th, by_cols; };

// One-dimensional transform out = B^T in for an even number of points, using what the generated B^T always looks like for
// the point sequence 0, +f, -f, +2f, -2f, ..., infinity (the host checks the matrix before it picks this path): row 0
// (point 0) is an even polynomial, the last row (infinity) an odd one, and the rows of +p and -p share their even
// coefficients and have opposite odd ones.  A pair of rows then costs one even and one odd dot product and two
// additions: half the multiply-adds of the dense product.
template <int A>
__device__ __forceinline__ void bt_apply_paired(const MatArg<A, A>& bt, const float (&in)[A], float (&out)[A])
{
    float e0 = bt.v[0][0] * in[0];
#pragma unroll
    for (int t = 2; t < A; t += 2) e0 = fmaf(bt.v[0][t], in[t], e0);
    out[0] = e0;
    float ol = bt.v[A - 1][1] * in[1];
#pragma unroll
    for (int t = 3; t < A; t += 2) ol = fmaf(bt.v[A - 1][t], in[t], ol);
    out[A - 1] = ol;
#pragma unroll
    for (int m = 1; m < A - 1; m += 2) {
        float e = bt.v[m][2] * in[2], o = bt.v[m][1] * in[1];
#pragma unroll
        for (int t = 4; t < A - 1; t += 2) e = fmaf(bt.v[m][t], in[t], e);
#pragma unroll
        for (int t = 3; t < A - 1; t += 2) o = fmaf(bt.v[m][t], in[t], o);
        out[m] = e + o;
        out[m + 1] = e - o;
    }
}

// One lane per (channel, tile); consecutive lanes are consecutive tiles, so every store of V is 256 contiguous bytes per
// wavefront and position.  Workgroups are handed out so that an XCD covers a contiguous range of (channel, tile) -- halo
// rows of neighbouring tiles meet in one L2.
// PAIRED: the B^T structure above holds (even A only).  WIDE: a tensor is too large for 32-bit byte offsets.
//
// What the kernel is made of matters as much as what it moves: alone, the loads of the largest layer take a third of
// its time, the stores a half, and the vector instructions that are neither (index arithmetic, a 64-bit address per
// load and store) most of the rest -- they do not hide behind the memory traffic.  So: tile coordinates come from
// multiplications, every load and store is addressed as a uniform base (scalar registers: tensor + row or position
// offset) plus one 32-bit lane offset computed once, and the paired transform halves the multiply-adds.
template <int A, bool BLOCKED, bool PAIRED, bool WIDE>
__global__ __launch_bounds__(256) void input_transform_kernel(WinoGeom g, InputMap mp, MatArg<A, A> bt,
                                                              const float* __restrict__ x,
                                                              float* __restrict__ V)
{
    using lane_off = typename std::conditional<WIDE, long long, unsigned>::type;
    const unsigned idx = xcd_contiguous(blockIdx.x, gridDim.x) * blockDim.x + threadIdx.x;       // < 2^31 (checked by the launcher)
    int c, p;
    lane_off vo;                                   // lane part of every V address, in floats
    if constexpr (BLOCKED) {
        // a wavefront owns 16 consecutive tiles x 4 consecutive channels = one 64-float block per position
        const unsigned rest = idx >> 6;
        const unsigned cq = fast_div(rest, mp.by_cols);            // mp.by_cols: groups of 16 tiles, ceil(P / 16)
        if (cq >= (unsigned)g.cchunks) return;
        const int pgrp = (int)(rest - cq * mp.by_cols.d);
        p = pgrp * 16 + (int)(idx & 15);
        c = (int)cq * 4 + (int)((idx >> 4) & 3);
        vo = ((lane_off)((long long)cq * A * g.pg + pgrp) << 6) + (lane_off)(idx & 63);
    } else {
        c = (int)fast_div(idx, mp.by_cols);                        // mp.by_cols: P
        if (c >= g.C) return;
        p = (int)(idx - (unsigned)c * mp.by_cols.d);
        vo = g.tiled ? (lane_off)(((long long)c * g.pb + (p >> 6)) * (A * A)) * 64 + (lane_off)(p & 63)
                     : (lane_off)((long long)c * g.ldp + p);
    }
    // element (a = i, b = j): row layout V[(i*A + j)][c][p]; blocked layout Vb[j][c/4][i][p/16][c%4][p%16]
    const long long stride_j = BLOCKED ? (long long)g.cchunks * A * g.pg * 64 : g.tiled ? 64ll : (long long)g.C * g.ldp;
    const long long stride_i = BLOCKED ? (long long)g.pg * 64 : stride_j * A;
    // in bytes for the narrow form: uniform 64-bit base + zero-extended 32-bit lane offset is an addressing mode of
    // the global memory instructions, a shifted 64-bit sum is two more vector instructions per access
    const lane_off vob = WIDE ? vo : vo * 4u;
    auto vstore = [&](int i, int j, float v) {
        float* base = V + (i * stride_i + j * stride_j);           // uniform: lives in scalar registers
        if constexpr (WIDE) base[vob] = v;
        else *reinterpret_cast<float*>(reinterpret_cast<char*>(base) + vob) = v;
    };
    if constexpr (BLOCKED) {
        if (p >= g.P || c >= g.C) {
            // padding of the blocked layout: the multiply stage reads it (against zero rows of U for
            // padded channels), so it must hold finite values whatever the memory held before
#pragma unroll 1
            for (int i = 0; i < A; ++i)
#pragma unroll 1
                for (int j = 0; j < A; ++j) vstore(i, j, 0.f);
            return;
        }
    }
    const unsigned t2 = fast_div((unsigned)p, mp.by_tw);
    const int tx = p - (int)t2 * g.tw;
    const unsigned img = fast_div(t2, mp.by_th);
    const int ty = (int)t2 - (int)img * g.th;
    const int y0 = ty * g.n - g.pad_h;
    const int x0 = tx * g.n - g.pad_w;
    // Loads.  A tile row is A consecutive floats: 16- and 8-byte loads at 4-byte alignment.  Tiles that hang over an edge
    // of the image take the very same loads -- rows above or below the image are clamped to its first or last row, columns
    // left or right of it simply read the neighbouring row or plane of the tensor -- and zero what lies outside afterwards:
    // with 22 tiles per row every wavefront holds edge tiles, and a separate element-by-element path for them (64 predicated
    // loads) would be issued by every wavefront.  Only a tile whose over-read would leave the tensor itself (the first rows of
    // the first plane, the last of the last) takes that path.
    const long long plane_ll = ((long long)img * g.C + c) * ((long long)g.H * g.W);
    const lane_off plane = (lane_off)plane_ll;
    const int ylo = y0 < 0 ? 0 : (y0 > g.H - 1 ? g.H - 1 : y0);
    const int yhi = y0 + A - 1 < 0 ? 0 : (y0 + A - 1 > g.H - 1 ? g.H - 1 : y0 + A - 1);
    const bool inside_tensor = plane_ll + (long long)ylo * g.W + x0 >= 0 &&
                               plane_ll + (long long)yhi * g.W + x0 + A <= (long long)g.N * g.C * g.H * g.W;
    const bool interior = (y0 >= 0) && (y0 + A <= g.H) && (x0 >= 0) && (x0 + A <= g.W);

    float d[A][A];
    if (inside_tensor) {
#pragma unroll
        for (int i = 0; i < A; ++i) {
            int iy = y0 + i;
            iy = iy < 0 ? 0 : (iy > g.H - 1 ? g.H - 1 : iy);
            // exact although x0 may be negative: the sum lies inside the tensor, and 32-bit arithmetic is modular
            const lane_off ro = plane + (lane_off)(iy * g.W + x0);
            const char* rp;
            if constexpr (WIDE) rp = reinterpret_cast<const char*>(x + ro);
            else rp = reinterpret_cast<const char*>(x) + ro * 4u;
            int j = 0;
#pragma unroll
            for (; j + 4 <= A; j += 4) {
                const Unaligned4 v = *reinterpret_cast<const Unaligned4*>(rp + j * 4);
                d[i][j] = v.x; d[i][j + 1] = v.y; d[i][j + 2] = v.z; d[i][j + 3] = v.w;
            }
            if (j + 2 <= A) {
                const Unaligned2 v = *reinterpret_cast<const Unaligned2*>(rp + j * 4);
                d[i][j] = v.x; d[i][j + 1] = v.y;
                j += 2;
            }
            if (j < A) d[i][j] = *reinterpret_cast<const float*>(rp + j * 4);
        }
        if (!interior) {
#pragma unroll
            for (int i = 0; i < A; ++i) {
                const bool rowok = (y0 + i >= 0) && (y0 + i < g.H);
#pragma unroll
                for (int j = 0; j < A; ++j) {
                    const bool ok = rowok && (x0 + j >= 0) && (x0 + j < g.W);
                    d[i][j] = ok ? d[i][j] : 0.f;
                }
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < A; ++i) {
            const int iy = y0 + i;
            const bool rowok = (iy >= 0) && (iy < g.H);
#pragma unroll
            for (int j = 0; j < A; ++j) {
                const int ix = x0 + j;
                const bool ok = rowok && (ix >= 0) && (ix < g.W);
                d[i][j] = ok ? x[plane_ll + (long long)iy * g.W + ix] : 0.f;
            }
        }
    }
    if constexpr (PAIRED) {
        // columns (t = B^T d, in place), then rows (v = t B), each row stored as soon as it exists
#pragma unroll
        for (int j = 0; j < A; ++j) {
            float in[A], out[A];
#pragma unroll
            for (int a = 0; a < A; ++a) in[a] = d[a][j];
            bt_apply_paired<A>(bt, in, out);
#pragma unroll
            for (int a = 0; a < A; ++a) d[a][j] = out[a];
        }
#pragma unroll
        for (int i = 0; i < A; ++i) {
            float out[A];
            bt_apply_paired<A>(bt, d[i], out);
#pragma unroll
            for (int j = 0; j < A; ++j) vstore(i, j, out[j]);
        }
    } else {
        // dense B^T, one row of t = B^T d at a time: row i of v needs row i of t only, so t never exists as a whole
#pragma unroll 1
        for (int i = 0; i < A; ++i) {
            float t[A];
#pragma unroll
            for (int j = 0; j < A; ++j) {
                float acc = 0.f;
#pragma unroll
                for (int a = 0; a < A; ++a) acc = fmaf(bt.v[i][a], d[a][j], acc);
                t[j] = acc;
            }
#pragma unroll
            for (int j = 0; j < A; ++j) {
                float acc = 0.f;
#pragma unroll
                for (int b = 0; b < A; ++b) acc = fmaf(t[b], bt.v[j][b], acc);
                vstore(i, j, acc);
            }
        }
    }
}

// ---------------------------------------------------------------- output: y = A^T m A + bias
struct OutputMap { FastDiv by_tw, by_th, by_p; };

// One-dimensional inverse transform out = init + A^T in for an even number of points (same point sequence as above; the
// host checks the matrix): the column of point 0 feeds only the first output, the column of infinity only the last,
// and the columns of +p and -p are equal in the even rows and opposite in the odd ones -- so a pair of inputs enters
// as its sum (even rows) and its difference (odd rows): half the multiply-adds of the dense product.
template <int NT, int A>
__device__ __forceinline__ void at_apply_paired(const MatArg<NT, A>& at, const float (&in)[A], float init, float (&out)[NT])
{
#pragma unroll
    for (int i = 0; i < NT; ++i) out[i] = init;
    out[0] = fmaf(at.v[0][0], in[0], out[0]);
    out[NT - 1] = fmaf(at.v[NT - 1][A - 1], in[A - 1], out[NT - 1]);
#pragma unroll
    for (int m = 1; m < A - 1; m += 2) {
        const float sum = in[m] + in[m + 1], dif = in[m] - in[m + 1];
#pragma unroll
        for (int i = 0; i < NT; ++i) out[i] = fmaf(at.v[i][m], (i & 1) ? dif : sum, out[i]);
    }
}

// One lane per (output channel, tile), consecutive lanes consecutive tiles.  As in the input transform, every load and
// store is a uniform base (tensor + position or row offset, scalar registers) plus one 32-bit lane offset in bytes.
// STREAM: M is larger than the last-level cache, so this (its last) read goes past the caches instead of
// evicting what the next kernel could still use; small M is read normally (it is still resident from the GEMM).
// VEC: how a tile row is stored -- 0: one float at a time; 1: pairs (n and W_o even, 8-byte aligned base);
// 2: one 16-byte store (n = 4, 4 | W_o, 16-byte aligned base).  A compile-time choice: with the choice made at run
// time the unused store paths stay in the kernel and cost 10 % of its time.
// PAIRED: the A^T structure above holds (even A only).  WIDE: M or y is too large for 32-bit byte offsets.
template <int NT, int A, bool STREAM, int VEC, bool PAIRED, bool WIDE>
__global__ __launch_bounds__(256) void output_transform_kernel(WinoGeom g, OutputMap mp, MatArg<NT, A> at,
                                                               const float* __restrict__ M,
                                                               const float* __restrict__ bias,
                                                               float* __restrict__ y)
{
    using lane_off = typename std::conditional<WIDE, long long, unsigned>::type;
    const unsigned idx = blockIdx.x * 256u + threadIdx.x;        // < 2^31 (checked by the launcher)
    const unsigned kk = fast_div(idx, mp.by_p);
    if (kk >= (unsigned)g.K) return;
    const unsigned p = idx - kk * mp.by_p.d;
    const unsigned t2 = fast_div(p, mp.by_tw);
    const int tx = (int)(p - t2 * (unsigned)g.tw);
    const unsigned img = fast_div(t2, mp.by_th);
    const int ty = (int)(t2 - img * (unsigned)g.th);

    const long long plane = g.tiled ? 64ll : (long long)g.K * g.ldp;
    const lane_off mo = g.tiled ? ((lane_off)kk * (lane_off)g.pb + (lane_off)(p >> 6)) * (lane_off)(A * A * 64) + (lane_off)(p & 63)
                                : (lane_off)kk * (lane_off)g.ldp + (lane_off)p;
    const lane_off mob = WIDE ? mo : mo * 4u;
    // All alpha^2 loads are issued before the first use: a wavefront then waits for memory once, not once per
    // row of m (the kernel is bound by that latency, not by registers: 4 or 8 wavefronts per SIMD make no difference).
    float m[A][A];
#pragma unroll
    for (int a = 0; a < A; ++a)
#pragma unroll
        for (int b = 0; b < A; ++b) {
            const float* base = M + (a * A + b) * plane;                       // uniform: lives in scalar registers
            const float* q;
            if constexpr (WIDE) q = base + mob;
            else q = reinterpret_cast<const float*>(reinterpret_cast<const char*>(base) + mob);
            m[a][b] = STREAM ? __builtin_nontemporal_load(q) : *q;
        }
    __builtin_amdgcn_sched_barrier(0);        // keep the compiler from sinking the loads between the multiply-adds
    // t = A^T m   (NT x A)
    float t[NT][A];
    if constexpr (PAIRED) {
#pragma unroll
        for (int b = 0; b < A; ++b) {
            float col[A], out[NT];
#pragma unroll
            for (int a = 0; a < A; ++a) col[a] = m[a][b];
            at_apply_paired<NT, A>(at, col, 0.f, out);
#pragma unroll
            for (int i = 0; i < NT; ++i) t[i][b] = out[i];
        }
    } else {
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
            for (int b = 0; b < A; ++b) t[i][b] = 0.f;
#pragma unroll
        for (int a = 0; a < A; ++a)
#pragma unroll
            for (int i = 0; i < NT; ++i)
#pragma unroll
                for (int b = 0; b < A; ++b) t[i][b] = fmaf(at.v[i][a], m[a][b], t[i][b]);
    }
    const float bv = bias ? bias[kk] : 0.f;
    const lane_off yo = (((lane_off)img * (lane_off)g.K + (lane_off)kk) * (lane_off)g.Ho + (lane_off)(ty * NT)) * (lane_off)g.Wo +
                        (lane_off)(tx * NT);
    const lane_off yob = WIDE ? yo : yo * 4u;
    const bool whole_w = tx * NT + NT <= g.Wo;      // the tile does not hang over the right edge
    // A lane owns NT consecutive floats of NT output rows.  Stores of one float per lane would touch
    // 64*NT*4/64 cache lines per instruction; pairs halve the number of store instructions.
#pragma unroll
    for (int i = 0; i < NT; ++i) {
        const int oy = ty * NT + i;
        float o[NT];
        if constexpr (PAIRED) {
            at_apply_paired<NT, A>(at, t[i], bv, o);
        } else {
#pragma unroll
            for (int j = 0; j < NT; ++j) {
                float acc = bv;
#pragma unroll
                for (int b = 0; b < A; ++b) acc = fmaf(t[i][b], at.v[j][b], acc);
                o[j] = acc;
            }
        }
        if (oy >= g.Ho) continue;
        float* rbase = y + (long long)i * g.Wo;                                // uniform
        float* row;
        if constexpr (WIDE) row = rbase + yob;
        else row = reinterpret_cast<float*>(reinterpret_cast<char*>(rbase) + yob);
        if constexpr (NT == 4 && VEC == 2) {
            {                         // 16-byte aligned tile rows, no ragged column
                *reinterpret_cast<float4*>(row) = make_float4(o[0], o[1], o[2], o[3]);
                continue;
            }
        }
        if constexpr (NT % 2 == 0 && VEC == 1) {
            // n and W_o even: a pair of columns lies inside the row or outside it, never across its end, so the
            // pairs need no 4-byte fallback (with one in the same loop the compiler turns every pair of every tile into
            // two predicated 4-byte stores: 180 instead of 156 us for F(6,3) on 128 x 128 x 256 x 16)
            {
                if (whole_w) {            // unconditional: the compiler joins the pairs of a row into 16-byte stores
#pragma unroll
                    for (int j = 0; j < NT; j += 2) *reinterpret_cast<float2*>(row + j) = make_float2(o[j], o[j + 1]);
                } else {
#pragma unroll
                    for (int j = 0; j < NT; j += 2)
                        if (tx * NT + j < g.Wo) *reinterpret_cast<float2*>(row + j) = make_float2(o[j], o[j + 1]);
                }
                continue;
            }
        }
#pragma unroll
        for (int j = 0; j < NT; ++j)
            if (tx * NT + j < g.Wo) row[j] = o[j];
    }
}

// Whether A^T (row-major NT x A) has the structure at_apply_paired relies on, exactly.
inline bool at_is_paired(const float* AT, int NT, int A)
{
    if (A % 2 || NT < 2) return false;
    for (int i = 1; i < NT; ++i) if (AT[i * A] != 0.f) return false;                       // point 0: first output only
    for (int i = 0; i < NT - 1; ++i) if (AT[i * A + A - 1] != 0.f) return false;           // infinity: last output only
    for (int m = 1; m < A - 1; m += 2)
        for (int i = 0; i < NT; ++i)
            if (AT[i * A + m + 1] != ((i & 1) ? -AT[i * A + m] : AT[i * A + m])) return false;
    return true;
}

// Whether B^T (row-major A x A) has the structure bt_apply_paired relies on, exactly.
inline bool bt_is_paired(const float* BT, int A)
{
    if (A % 2) return false;
    for (int t = 1; t < A; t += 2) if (BT[t] != 0.f) return false;                         // row 0: even
    for (int t = 0; t < A; t += 2) if (BT[(A - 1) * A + t] != 0.f) return false;           // last row: odd
    for (int m = 1; m < A - 1; m += 2) {
        if (BT[m * A] != 0.f || BT[m * A + A - 1] != 0.f || BT[(m + 1) * A] != 0.f || BT[(m + 1) * A + A - 1] != 0.f) return false;
        for (int t = 1; t < A - 1; ++t)
            if (BT[(m + 1) * A + t] != ((t & 1) ? -BT[m * A + t] : BT[m * A + t])) return false;
    }
    return true;
}

template <int A>
hipError_t launch_input_t(const WinoGeom& g, const float* BT, const float* x, float* V, hipStream_t s)
{
    MatArg<A, A> m;
    for (int i = 0; i < A; ++i)
        for (int j = 0; j < A; ++j) m.v[i][j] = BT[i * A + j];
    // V is stored normally even when it is far larger than the caches: stores that go past them make this
    // kernel 25-35 % faster run alone but slower in sequence -- normal stores park about half of V in the 256 MB
    // last-level cache, its write-back overlaps the matrix-core-bound GEMM, and the GEMM finds that half there.
    const long long cols = g.blocked ? (g.P + 15) / 16 : g.P;
    const long long lanes = g.blocked ? (long long)g.cchunks * cols * 64 : (long long)g.C * cols;
    if (lanes <= 0 || lanes + 256 >= (1ll << 31)) return hipErrorInvalidValue;
    // Fewer wavefronts per CU than the registers allow: the kernel is bound by the memory system, and past 10 to 16 resident
    // wavefronts per CU more concurrent store streams only thrash it (10 % slower at 24).  LDS the kernel never touches is
    // the lever: a workgroup that asks for 1/n of a CU's 160 KB leaves room for n of them.  A count that is not a multiple
    // of four takes workgroups of two wavefronts (row layouts only: the blocked layout wants four adjacent units per workgroup).
    int bs = 256;
    size_t cap_lds = 0;
    if (g.itx_waves >= 8 && g.itx_waves <= 32) {
        if (g.itx_waves % 4 != 0 && !g.blocked) bs = 128;
        const int wgs = g.itx_waves / (bs / 64);
        if (wgs >= 3) cap_lds = ((size_t)160 * 1024 / wgs - 1024) / 256 * 256;
    }
    const unsigned blocks = (unsigned)((lanes + bs - 1) / bs);
    InputMap mp{make_fastdiv((unsigned)g.tw), make_fastdiv((unsigned)g.th), make_fastdiv((unsigned)cols)};
    // 32-bit byte offsets: the input, one position plane of V (row layout) or one slab of V (blocked) below 4 GiB
    const long long in_elems = (long long)g.N * g.C * g.H * g.W;
    const long long v_elems = g.blocked ? (long long)g.cchunks * A * g.pg * 64 : (long long)g.C * g.ldp * (g.tiled ? A * A : 1);
    const bool wide = in_elems >= (1ll << 30) || v_elems >= (1ll << 30);
    const bool paired = bt_is_paired(BT, A);
    const dim3 grid(blocks), block(bs);
    auto launch = [&](auto kernel) { hipLaunchKernelGGL(kernel, grid, block, cap_lds, s, g, mp, m, x, V); };
    auto pick = [&](auto blocked_c, auto wide_c) {
        constexpr bool B = decltype(blocked_c)::value, W = decltype(wide_c)::value;
        if constexpr (A % 2 == 0) {
            if (paired) { launch(input_transform_kernel<A, B, true, W>); return; }
        }
        launch(input_transform_kernel<A, B, false, W>);
    };
    if (g.blocked) { if (wide) pick(std::true_type{}, std::true_type{}); else pick(std::true_type{}, std::false_type{}); }
    else           { if (wide) pick(std::false_type{}, std::true_type{}); else pick(std::false_type{}, std::false_type{}); }
    return hipGetLastError();
}

template <int NT, int A>
hipError_t launch_output_t(const WinoGeom& g, const float* AT, const float* M, const float* bias,
                           float* y, hipStream_t s)
{
    MatArg<NT, A> m;
    for (int i = 0; i < NT; ++i)
        for (int j = 0; j < A; ++j) m.v[i][j] = AT[i * A + j];
    const long long total = (long long)g.K * g.P;
    if (total <= 0 || total + 256 >= (1ll << 31)) return hipErrorInvalidValue;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    // 8-byte stores need every tile row start 8-byte aligned: even n, even W_o, aligned base
    int vec2 = (NT % 2 == 0) && (g.Wo % 2 == 0) && ((reinterpret_cast<uintptr_t>(y) & 7u) == 0);
    if (NT == 4 && (g.Wo % 4 == 0) && ((reinterpret_cast<uintptr_t>(y) & 15u) == 0)) vec2 = 2;   // whole-tile float4 rows
    // 256 MB of last-level cache on this part; well above half of it nothing of M survives until it is read
    const bool stream = (double)A * A * g.K * g.ldp * sizeof(float) > 160e6;
    // 32-bit byte offsets: what a lane adds to a uniform base -- all of M in the tiled layout, one position plane of it in
    // the row layout, all of y -- stays below 4 GiB
    const long long m_lane_elems = (long long)g.K * g.ldp * (g.tiled ? A * A : 1);
    const long long y_elems = (long long)g.N * g.K * g.Ho * g.Wo;
    const bool wide = m_lane_elems >= (1ll << 30) || y_elems >= (1ll << 30);
    const bool paired = at_is_paired(AT, NT, A);
    OutputMap mp{make_fastdiv((unsigned)g.tw), make_fastdiv((unsigned)g.th), make_fastdiv((unsigned)g.P)};
    auto launch = [&](auto kernel) { hipLaunchKernelGGL(kernel, dim3(blocks), dim3(256), 0, s, g, mp, m, M, bias, y); };
    // a tensor that needs 64-bit offsets is far larger than the caches: the wide form exists for streamed reads only
    auto pick = [&](auto vec_c) {
        constexpr int V = decltype(vec_c)::value;
        if constexpr (A % 2 == 0) {
            if (paired) {
                if (wide) launch(output_transform_kernel<NT, A, true, V, true, true>);
                else if (stream) launch(output_transform_kernel<NT, A, true, V, true, false>);
                else launch(output_transform_kernel<NT, A, false, V, true, false>);
                return;
            }
        }
        if (wide) launch(output_transform_kernel<NT, A, true, V, false, true>);
        else if (stream) launch(output_transform_kernel<NT, A, true, V, false, false>);
        else launch(output_transform_kernel<NT, A, false, V, false, false>);
    };
    if constexpr (NT == 4) {
        if (vec2 == 2) { pick(std::integral_constant<int, 2>{}); return hipGetLastError(); }
    }
    if constexpr (NT % 2 == 0) {
        if (vec2) { pick(std::integral_constant<int, 1>{}); return hipGetLastError(); }
    }
    pick(std::integral_constant<int, 0>{});
    return hipGetLastError();
}

bool geom_ok(const WinoGeom& g)
{
    if (g.N <= 0 || g.C <= 0 || g.H <= 0 || g.W <= 0 || g.K <= 0) return false;
    if (g.n < 2 || g.k < 2 || g.k > kMaxK || g.alpha != g.n + g.k - 1 || g.alpha > kMaxAlphaT) return false;
    if (g.nw != g.n || g.kw != g.k || g.alpha_w != g.alpha) return false;      // square kernels only here
    if (g.Ho != g.H + 2 * g.pad_h - g.k + 1 || g.Wo != g.W + 2 * g.pad_w - g.k + 1) return false;
    if (g.Ho <= 0 || g.Wo <= 0) return false;
    if (g.th != (g.Ho + g.n - 1) / g.n || g.tw != (g.Wo + g.n - 1) / g.n) return false;
    if ((long long)g.P != (long long)g.N * g.th * g.tw) return false;
    if (g.blocked) {
        if ((long long)g.cchunks * 4 < g.C || (long long)g.kg * 16 < g.K || (long long)g.pg * 16 < g.P) return false;
    } else if (g.ldp < g.P || g.ldk < g.K || (g.tiled && ((long long)g.pb * 64 != g.ldp))) {
        return false;
    }
    // every per-plane element count must fit the 32-bit tile arithmetic used in the kernels
    if ((long long)g.C * g.ldp >= (1ll << 31) || (long long)g.K * g.ldp >= (1ll << 31)) return false;
    if ((long long)g.H * g.W >= (1ll << 31)) return false;
    return true;
}

}  // namespace

bool winograd_kernels_available(int n, int k)
{
    const int a = n + k - 1;
    return n >= 2 && n <= 8 && k >= 2 && k <= kMaxK && a <= kMaxAlphaT;
}

hipError_t launch_filter_transform(const WinoGeom& g, const float* G, const float* w, float* U, hipStream_t s)
{
    if (!geom_ok(g) || !G || !w || !U) return hipErrorInvalidValue;
    FilterMat m;
    for (int i = 0; i < kMaxAlphaT; ++i)
        for (int j = 0; j < kMaxK; ++j) m.g[i][j] = (i < g.alpha && j < g.k) ? G[i * g.k + j] : 0.f;
    const long long total = (long long)g.K * g.C;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    switch (g.k) {
#define MNN_FILTER(KT_) case KT_: hipLaunchKernelGGL(filter_transform_kernel<KT_>, dim3(blocks), dim3(256), 0, s, g, m, w, U); break;
        MNN_FILTER(2) MNN_FILTER(3) MNN_FILTER(4) MNN_FILTER(5) MNN_FILTER(6) MNN_FILTER(7)
#undef MNN_FILTER
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_input_transform(const WinoGeom& g, const float* BT, const float* x, float* V, hipStream_t s)
{
    if (!geom_ok(g) || !BT || !x || !V) return hipErrorInvalidValue;
    switch (g.alpha) {
#define MNN_CASE(A) case A: return launch_input_t<A>(g, BT, x, V, s);
        MNN_CASE(3) MNN_CASE(4) MNN_CASE(5) MNN_CASE(6) MNN_CASE(7) MNN_CASE(8)
        MNN_CASE(9) MNN_CASE(10)
#undef MNN_CASE
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_output_transform(const WinoGeom& g, const float* AT, const float* M, const float* bias,
                                   float* y, hipStream_t s)
{
    if (!geom_ok(g) || !AT || !M || !y) return hipErrorInvalidValue;
    if (!winograd_kernels_available(g.n, g.k)) return hipErrorInvalidValue;
#define MNN_NK(NN, KK) \
    if (g.n == NN && g.k == KK) return launch_output_t<NN, NN + KK - 1>(g, AT, M, bias, y, s);
    // every (n, k) with 2 <= n <= 8, 2 <= k <= 7 and n + k - 1 <= 10
    MNN_NK(2, 2) MNN_NK(3, 2) MNN_NK(4, 2) MNN_NK(5, 2) MNN_NK(6, 2) MNN_NK(7, 2) MNN_NK(8, 2)
    MNN_NK(2, 3) MNN_NK(3, 3) MNN_NK(4, 3) MNN_NK(5, 3) MNN_NK(6, 3) MNN_NK(7, 3) MNN_NK(8, 3)
    MNN_NK(2, 4) MNN_NK(3, 4) MNN_NK(4, 4) MNN_NK(5, 4) MNN_NK(6, 4) MNN_NK(7, 4)
    MNN_NK(2, 5) MNN_NK(3, 5) MNN_NK(4, 5) MNN_NK(5, 5) MNN_NK(6, 5)
    MNN_NK(2, 6) MNN_NK(3, 6) MNN_NK(4, 6) MNN_NK(5, 6)
    MNN_NK(2, 7) MNN_NK(3, 7) MNN_NK(4, 7)
#undef MNN_NK
    return hipErrorInvalidValue;
}

}  // namespace mnnconv
