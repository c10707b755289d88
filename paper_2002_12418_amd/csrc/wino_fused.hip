// Winograd-domain matrix multiplication with the inverse transform fused in
// (Section 3.3.1 of the MNN paper: the channel sum of Hadamard products becomes
// one matrix product per transformed position, followed by Y = A^T [.] A).
// The product tensor M is never stored.
//
// Structure.  The inverse transform is separable,
//     Y = sum_b (A^T m[:, b]) (x) A^T[:, b],      m[a][b] = M_(a,b)[k][p],
// so the alpha x alpha positions are processed one COLUMN b at a time: for a
// column the workgroup runs the complete channel reduction of its alpha
// positions (a, b), a = 0..alpha-1, on the matrix cores, then folds the alpha
// accumulators of every (k, p) pair into that pair's n x n output registers and
// reuses the accumulators for the next column.  For one (k, p) the alpha values
// sit in the same lane and register slot of alpha MFMA tiles, so the fold is
// plain per-lane arithmetic.  Registers per 16x16 tile: 4 alpha accumulators +
// 4 n^2 outputs (instead of 4 alpha^2), which leaves room for two wavefronts
// per SIMD; the second one hides barrier and LDS latency of the first.
//
// Operand layout ("MFMA-native", the counterpart of the paper's layout
// re-ordering for SIMD).  Both operands are stored in blocks of 4 channels x 16
// columns = 64 contiguous floats, exactly one v_mfma_f32_16x16x4_f32 operand
// (lane l holds channel l/16, column l%16), ordered so that the stream a
// workgroup consumes is sequential:
//     Ub[b][c/4][a][k/16][c%4][k%16]      (K padded to kg*16 columns)
//     Vb[b][c/4][a][p/16][c%4][p%16]      (P padded to pg*16 columns)
// with the channel count padded to a whole number of chunks.  A chunk (BKG
// 4-channel groups x alpha positions) is copied global -> LDS as is by
// global_load_lds_dwordx4, without passing through registers, while the MFMAs
// of the previous chunk run; every MFMA operand is then one conflict-free
// ds_read_b32 of 64 consecutive floats.
#include <hip/hip_runtime.h>
#include <map>
#include <mutex>
#include <utility>
#include "kernels.hpp"
#include "xcd_remap.hpp"

namespace mnnconv {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void glb_void;

// s_waitcnt vmcnt(N) for a compile-time N (0..63): bits [3:0] and [15:14] hold vmcnt on gfx9
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N <= 63, "vmcnt range");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

template <int A, int NT_, int WTM, int WTN, int WM, int WN, int BKG, int NS>
__global__ __launch_bounds__(WM * WN * 64, (WM * WN > 8 ? 1 : 2)) void wino_fused_kernel(WinoGeom g, MatArg<NT_, A> at,
                                                                  const float* __restrict__ Ub,
                                                                  const float* __restrict__ Vb,
                                                                  const float* __restrict__ bias,
                                                                  float* __restrict__ y, int kblocks, int nch,
                                                                  int vec_store, int pb0)
{
    constexpr int NW = WM * WN;
    constexpr int MG = WM * WTM;              // 16-row groups of the K block
    constexpr int PG = WN * WTN;              // 16-column groups of the tile block
    constexpr int UQ = BKG * A * MG / 4;      // wavefront-wide 1 KiB copies per chunk
    constexpr int VQ = BKG * A * PG / 4;
    static_assert((BKG * A * MG) % 4 == 0 && (BKG * A * PG) % 4 == 0, "chunk must be whole KiB copies");
    constexpr int JU = (UQ + NW - 1) / NW;    // copies per wavefront per chunk (every wavefront issues all of them)
    constexpr int JV = (VQ + NW - 1) / NW;
    constexpr int LPW = JU + JV;
    static_assert(NS >= 2 && NS <= 4 && (NS - 2) * LPW <= 63, "stage count");

    // NS stages of the operand blocks in a ring.  They are separate objects, selected by a stage
    // index that is a compile-time constant wherever it is used: the compiler then knows that the
    // LDS reads of one stage cannot touch the stage a copy is still writing, and does not stall
    // the reads on the copies in flight.
    __shared__ __attribute__((aligned(16))) float Us0[UQ * 256];
    __shared__ __attribute__((aligned(16))) float Us1[UQ * 256];
    __shared__ __attribute__((aligned(16))) float Us2[NS > 2 ? UQ * 256 : 4];
    __shared__ __attribute__((aligned(16))) float Us3[NS > 3 ? UQ * 256 : 4];
    __shared__ __attribute__((aligned(16))) float Vs0[VQ * 256];
    __shared__ __attribute__((aligned(16))) float Vs1[VQ * 256];
    __shared__ __attribute__((aligned(16))) float Vs2[NS > 2 ? VQ * 256 : 4];
    __shared__ __attribute__((aligned(16))) float Vs3[NS > 3 ? VQ * 256 : 4];
    auto ustage = [&](int st) -> float* { return st == 0 ? Us0 : st == 1 ? Us1 : st == 2 ? Us2 : Us3; };
    auto vstage = [&](int st) -> float* { return st == 0 ? Vs0 : st == 1 ? Vs1 : st == 2 ? Vs2 : Vs3; };

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;
    // every XCD gets a contiguous range of the grid, so that the K blocks of one tile block (K blocks fastest)
    // read their common V block through one L2
    const int wg = (int)xcd_contiguous(blockIdx.x, gridDim.x);
    const int kb = wg % kblocks;
    const int pb = pb0 + wg / kblocks;         // pb0: first tile block of this launch (a launch may cover a range)

    const float* __restrict__ Up = Ub + (long long)kb * MG * 64;
    const float* __restrict__ Vp = Vb + (long long)pb * PG * 64;
    const long long u_step = (long long)BKG * A * g.kg * 64;   // floats per chunk in the global stream
    const long long v_step = (long long)BKG * A * g.pg * 64;

    // Per-lane source offsets of this wavefront's copies inside a chunk: LDS image [ccl][a][group][64].
    // Copy j of wavefront w is piece j * NW + w.  With two stages every wait is for all copies, so a wavefront simply
    // skips the pieces past the end (a wavefront-uniform branch); with more stages the waits count copies, every
    // wavefront must have exactly LPW of them in flight per chunk, and a piece past the end repeats an earlier one
    // (same bytes to the same place).
    constexpr bool EXACT = (NS == 2);
    int uo[JU], vo[JV], uq[JU], vq[JV];
#pragma unroll
    for (int j = 0; j < JU; ++j) {
        uq[j] = EXACT ? j * NW + wave : (j * NW + wave) % UQ;
        const int s = (uq[j] % UQ) * 64 + lane;              // 16-byte slot
        uo[j] = (s / (MG * 16)) * g.kg * 64 + (s % (MG * 16)) * 4;
    }
#pragma unroll
    for (int j = 0; j < JV; ++j) {
        vq[j] = EXACT ? j * NW + wave : (j * NW + wave) % VQ;
        const int s = (vq[j] % VQ) * 64 + lane;
        vo[j] = (s / (PG * 16)) * g.pg * 64 + (s % (PG * 16)) * 4;
    }

    // Global memory -> LDS without passing through registers (global_load_lds_dwordx4): lane l of a
    // wavefront-wide copy writes LDS bytes [base + 16 l, base + 16 l + 16).
    auto issue = [&](int t, int st) {
        const float* ug = Up + t * u_step;
        const float* vg = Vp + t * v_step;
#pragma unroll
        for (int j = 0; j < JU; ++j)
            if (!EXACT || (j + 1) * NW <= UQ || uq[j] < UQ)
                __builtin_amdgcn_global_load_lds((glb_void*)(ug + uo[j]), (lds_void*)(ustage(st) + uq[j] * 256), 16, 0, 0);
#pragma unroll
        for (int j = 0; j < JV; ++j)
            if (!EXACT || (j + 1) * NW <= VQ || vq[j] < VQ)
                __builtin_amdgcn_global_load_lds((glb_void*)(vg + vo[j]), (lds_void*)(vstage(st) + vq[j] * 256), 16, 0, 0);
    };

    floatx4 acc[A][WTM][WTN];
    float Y[WTM][WTN][4][NT_][NT_];
#pragma unroll
    for (int a = 0; a < A; ++a)
#pragma unroll
        for (int i = 0; i < WTM; ++i)
#pragma unroll
            for (int j = 0; j < WTN; ++j) acc[a][i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int ii = 0; ii < NT_; ++ii)
#pragma unroll
                    for (int jj = 0; jj < NT_; ++jj) Y[i][j][r][ii][jj] = 0.f;

    // The operands of position idx + 1 are read from LDS before the MFMAs of position idx are issued, so that a
    // wavefront's matrix instructions follow each other without an LDS round trip between them.
    auto multiply = [&](int st) {
        const float* us = ustage(st) + (wm * WTM) * 64 + lane;
        const float* vs = vstage(st) + (wn * WTN) * 64 + lane;
        constexpr int NP = BKG * A;            // (channel group, position) pairs of a chunk, in LDS order
        float av[2][WTM], bv[2][WTN];
#pragma unroll
        for (int i = 0; i < WTM; ++i) av[0][i] = us[i * 64];
#pragma unroll
        for (int j = 0; j < WTN; ++j) bv[0][j] = vs[j * 64];
#pragma unroll
        for (int idx = 0; idx < NP; ++idx) {
            const int cur = idx & 1, nxt = cur ^ 1;
            if (idx + 1 < NP) {
#pragma unroll
                for (int i = 0; i < WTM; ++i) av[nxt][i] = us[((idx + 1) * MG + i) * 64];
#pragma unroll
                for (int j = 0; j < WTN; ++j) bv[nxt][j] = vs[((idx + 1) * PG + j) * 64];
            }
            __builtin_amdgcn_sched_barrier(0);     // the scheduler would otherwise pair each read with its own MFMA again
            const int a = idx % A;
#pragma unroll
            for (int i = 0; i < WTM; ++i)
#pragma unroll
                for (int j = 0; j < WTN; ++j)
                    acc[a][i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[cur][i], bv[cur][j], acc[a][i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Y += (A^T m[:, b]) (x) A^T[:, b] for every (k, p) pair this lane owns; accumulators restart at 0.
    auto fold = [&](int b) {
        float atb[NT_];
#pragma unroll
        for (int jj = 0; jj < NT_; ++jj) atb[jj] = at.v[jj][b];
#pragma unroll
        for (int i = 0; i < WTM; ++i)
#pragma unroll
            for (int j = 0; j < WTN; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
#pragma unroll
                    for (int ii = 0; ii < NT_; ++ii) {
                        float t = 0.f;
#pragma unroll
                        for (int a = 0; a < A; ++a) t = fmaf(at.v[ii][a], acc[a][i][j][r], t);
#pragma unroll
                        for (int jj = 0; jj < NT_; ++jj) Y[i][j][r][ii][jj] = fmaf(t, atb[jj], Y[i][j][r][ii][jj]);
                    }
                }
#pragma unroll
        for (int a = 0; a < A; ++a)
#pragma unroll
            for (int i = 0; i < WTM; ++i)
#pragma unroll
                for (int j = 0; j < WTN; ++j) acc[a][i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    };

    // Chunk steps t = 0 .. T-1: column b = t / nch, chunk t % nch; stage t % NS.  While step t is
    // multiplied, the copies of steps t+1 .. t+NS-1 are in flight.
    const int T = A * nch;
    int next_fold = nch - 1;                   // step after which column b is complete
    int b = 0;
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
        if (s < T) issue(s, s);
    if (NS - 1 <= T) wait_vmcnt<(NS - 2) * LPW>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();

    for (int t0 = 0; t0 < T; t0 += NS) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {          // stage index is static inside the unrolled body
            const int t = t0 + s;
            if (t < T) {
                // stage (s + NS - 1) % NS was read by step t - 1, which every wavefront has finished
                const bool more = t + NS - 1 < T;
                if (more) issue(t + NS - 1, (s + NS - 1) % NS);
                multiply(s);
                if (t == next_fold) {
                    fold(b);
                    ++b;
                    next_fold += nch;
                }
                // step t + 1 must have landed; the NS - 2 younger chunks may stay in flight
                // (a plain s_barrier: the copies are tracked by vmcnt above, and the LDS reads of this
                // step were consumed by its MFMAs, so no memory fence is needed here)
                if (more) wait_vmcnt<(NS - 2) * LPW>(); else wait_vmcnt<0>();
                __builtin_amdgcn_s_barrier();
            }
        }
    }

    // ---- write the n x n outputs.  In a 16x16 MFMA tile lane l, slot r holds row 4*(l/16) + r, column l%16.
    const int tiles_per_img = g.th * g.tw;
#pragma unroll
    for (int j = 0; j < WTN; ++j) {
        const int p = (pb * PG + wn * WTN + j) * 16 + (lane & 15);
        if (p >= g.P) continue;
        const int img = p / tiles_per_img;
        const int trem = p % tiles_per_img;
        const int ty = trem / g.tw, tx = trem % g.tw;
#pragma unroll
        for (int i = 0; i < WTM; ++i) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int kk = (kb * MG + wm * WTM + i) * 16 + 4 * (lane >> 4) + r;
                if (kk >= g.K) continue;
                const float bv = bias ? bias[kk] : 0.f;
                float* yp = y + ((long long)img * g.K + kk) * g.Ho * g.Wo + (long long)(ty * NT_) * g.Wo + tx * NT_;
#pragma unroll
                for (int ii = 0; ii < NT_; ++ii) {
                    if (ty * NT_ + ii >= g.Ho) continue;
                    float* row = yp + (long long)ii * g.Wo;
                    if constexpr (NT_ == 4) {
                        if (vec_store) {
                            *reinterpret_cast<float4*>(row) = make_float4(Y[i][j][r][ii][0] + bv, Y[i][j][r][ii][1] + bv,
                                                                           Y[i][j][r][ii][2] + bv, Y[i][j][r][ii][3] + bv);
                            continue;
                        }
                    }
                    if constexpr (NT_ == 2) {
                        if (vec_store) {
                            *reinterpret_cast<float2*>(row) = make_float2(Y[i][j][r][ii][0] + bv, Y[i][j][r][ii][1] + bv);
                            continue;
                        }
                    }
#pragma unroll
                    for (int jj = 0; jj < NT_; ++jj)
                        if (tx * NT_ + jj < g.Wo) row[jj] = Y[i][j][r][ii][jj] + bv;
                }
            }
        }
    }
}

// Range of one launch, in tile blocks of the configuration: [first, first + count); count < 0 = to the end.
// resident != nullptr: only report how many workgroups of this configuration the device holds at once.
struct FusedRange { int first = 0, count = -1; int* resident = nullptr; };

template <int NT_, int K_, int WTM, int WTN, int WM, int WN, int BKG, int NS>
hipError_t launch_fused_t(const WinoGeom& g, const float* AT, const float* Ub, const float* Vb, const float* bias,
                          float* y, hipStream_t s, const FusedRange& r)
{
    constexpr int A = NT_ + K_ - 1;
    constexpr int KB = WM * WTM * 16, PB = WN * WTN * 16;
    auto kernel = wino_fused_kernel<A, NT_, WTM, WTN, WM, WN, BKG, NS>;
    if (r.resident) {
        int per_cu = 0, dev = 0, cus = 0;
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, WM * WN * 64, 0);
        if (e == hipSuccess) e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        *r.resident = per_cu * cus;
        return hipSuccess;
    }
    // the kernel copies whole blocks and whole chunks without bounds checks: the padded extents must cover them
    const int kblocks = (g.K + KB - 1) / KB;
    const int pblocks = (g.P + PB - 1) / PB;
    if (kblocks * (KB / 16) > g.kg || pblocks * (PB / 16) > g.pg) return hipErrorInvalidValue;
    if (g.cchunks % BKG != 0 || g.cchunks * 4 < g.C) return hipErrorInvalidValue;
    const int count = r.count < 0 ? pblocks - r.first : r.count;
    if (r.first < 0 || count < 0 || r.first + count > pblocks) return hipErrorInvalidValue;
    if (count == 0) return hipSuccess;
    if ((long long)kblocks * count >= (1ll << 31)) return hipErrorInvalidValue;
    MatArg<NT_, A> m;
    for (int i = 0; i < NT_; ++i)
        for (int j = 0; j < A; ++j) m.v[i][j] = AT[i * A + j];
    // vector stores need every tile row start 16/8-byte aligned: W_o a multiple of n and an aligned base
    const bool vec = (NT_ == 4 || NT_ == 2) && (g.Wo % NT_ == 0) && ((reinterpret_cast<uintptr_t>(y) & 15u) == 0);
    hipLaunchKernelGGL(kernel, dim3((unsigned)(kblocks * count)), dim3(WM * WN * 64), 0, s, g, m, Ub, Vb, bias, y, kblocks,
                       g.cchunks / BKG, vec ? 1 : 0, r.first);
    return hipGetLastError();
}

// registers per lane: 4*alpha accumulators + 4*n^2 outputs per 16x16 tile
// 4-channel groups per chunk: a stage of both operands is BKG * alpha * (MG + PG) blocks of 256 bytes,
// 16 to 24 KiB for 32 x 32 blocks and twice that for 64 x 64
constexpr int bkg_for(int alpha) { return alpha <= 6 ? 4 : 2; }
// Stages of the operand ring.  Two: one chunk being multiplied, one in flight.  A third stage (or a fourth) buys
// less than the workgroups per CU it costs: at 16 KiB per stage, two stages let five 32 x 32 workgroups share a CU
// instead of three (F(2,7) C = 64: 0.346 -> 0.320 ms, F(4,5) C = 128: 0.111 -> 0.103 ms).
constexpr int kStages = 2;

constexpr bool fits_big(int n, int k) { return (2 * (4 * (n + k - 1) + 4 * n * n)) <= 192; }
// 64 x 64 blocks as sixteen wavefronts of one tile each (four per SIMD: 128 registers), for the tiles whose two-tile
// wavefronts do not fit
constexpr bool fits_big16(int n, int k) { return !fits_big(n, k) && 4 * (n + k - 1) + 4 * n * n <= 108; }
// one 16x16 tile per wavefront must leave room for two wavefronts per SIMD (256 registers each)
constexpr bool fits_small(int n, int k) { return 4 * (n + k - 1) + 4 * n * n <= 230; }

}  // namespace

bool wino_fused_available(int n, int k)
{
    const int a = n + k - 1;
    return n >= 2 && k >= 2 && a <= kMaxAlphaT && fits_small(n, k) && winograd_kernels_available(n, k);
}

bool wino_fused_has_big_block(int n, int k) { return wino_fused_available(n, k) && (fits_big(n, k) || fits_big16(n, k)); }

namespace {

hipError_t dispatch_fused(const WinoGeom& g, int config, const float* AT, const float* Ub, const float* Vb, const float* bias,
                          float* y, hipStream_t s, const FusedRange& r)
{
#define MNN_FUSED(NN, KK)                                                                       \
    if (g.n == NN && g.k == KK) {                                                                \
        if constexpr (fits_big(NN, KK)) {                                                        \
            if (config == 1) return launch_fused_t<NN, KK, 2, 1, 2, 4, bkg_for(NN + KK - 1), kStages>(g, AT, Ub, Vb, bias, y, s, r);  \
        }                                                                                        \
        if constexpr (fits_big16(NN, KK)) {                                                      \
            if (config == 1) return launch_fused_t<NN, KK, 1, 1, 4, 4, bkg_for(NN + KK - 1), kStages>(g, AT, Ub, Vb, bias, y, s, r);  \
        }                                                                                        \
        return launch_fused_t<NN, KK, 1, 1, 2, 2, bkg_for(NN + KK - 1), kStages>(g, AT, Ub, Vb, bias, y, s, r);                       \
    }
    MNN_FUSED(2, 2) MNN_FUSED(3, 2) MNN_FUSED(4, 2) MNN_FUSED(5, 2) MNN_FUSED(6, 2) MNN_FUSED(7, 2)
    MNN_FUSED(2, 3) MNN_FUSED(3, 3) MNN_FUSED(4, 3) MNN_FUSED(5, 3) MNN_FUSED(6, 3)
    MNN_FUSED(2, 4) MNN_FUSED(3, 4) MNN_FUSED(4, 4) MNN_FUSED(5, 4)
    MNN_FUSED(2, 5) MNN_FUSED(3, 5) MNN_FUSED(4, 5)
    MNN_FUSED(2, 6) MNN_FUSED(3, 6)
    MNN_FUSED(2, 7)
    // alpha = 9 and 10 where the n x n outputs still fit the registers
    MNN_FUSED(6, 4) MNN_FUSED(5, 5) MNN_FUSED(6, 5) MNN_FUSED(4, 6) MNN_FUSED(5, 6) MNN_FUSED(3, 7) MNN_FUSED(4, 7)
#undef MNN_FUSED
    return hipErrorInvalidValue;
}

// workgroups of the 64 x 64 configuration the device holds at once, per (n, k); 0 = not asked yet
std::mutex g_resident_mu;
std::map<std::pair<int, int>, int> g_resident64;

}  // namespace

namespace {

// How many tile blocks of 64 the 64 x 64 configuration takes (the rest goes to 32 x 32 workgroups): all of them, or
// those that fill whole rounds of resident workgroups when the last round would be at most 60 % full.
hipError_t big_block_share(const WinoGeom& g, int* p_big)
{
    int resident = 0;
    {
        std::lock_guard<std::mutex> lk(g_resident_mu);
        int& slot = g_resident64[{g.n, g.k}];
        if (slot == 0) {
            FusedRange q;
            q.resident = &slot;
            const hipError_t e = dispatch_fused(g, 1, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, q);
            if (e != hipSuccess) { slot = 0; return e; }
        }
        resident = slot;
    }
    const int kblocks = (g.K + 63) / 64, pblocks = (g.P + 63) / 64;
    const long long total = (long long)kblocks * pblocks;
    *p_big = pblocks;
    if (resident > 0 && total > resident) {
        const long long rounds = total / resident;
        const long long last = total - rounds * resident;  // workgroups of the last, partial round
        if (last > 0 && last * 10 <= (long long)resident * 6) *p_big = (int)(rounds * resident / kblocks);
    }
    return hipSuccess;
}

}  // namespace

// config 0: 32 channels x 32 tiles per workgroup (4 wavefronts, one 16x16 tile each);
// config 1: 64 channels x 64 tiles: 8 wavefronts of two tiles each along K where two tiles fit 256 registers, else 16
// wavefronts of one tile each where one tile fits 128 (F(4,6), F(4,7): the kernel is paced by what a CU can copy
// from L2 per cycle, and the larger block halves the bytes per multiply -- 190 -> 173 us for F(4,7) on 16 x 64 x 112 x 112
// although its 196 workgroups, one per CU, leave 60 CUs idle).
//
// The 64 x 64 workgroups are few and long (two per CU): a grid of 1.5 times what the device holds runs as two
// rounds, the second half empty.  When the last round would be at most 60 % full, config 1 therefore covers only the
// tile blocks that fill whole rounds and the rest of the tiles is launched as 32 x 32 workgroups, which are
// short and pack five to a CU (same operands, same order of additions: the same bits).
hipError_t launch_wino_fused(const WinoGeom& g, int config, const float* AT, const float* Ub, const float* Vb,
                             const float* bias, float* y, hipStream_t s)
{
    if (!AT || !Ub || !Vb || !y) return hipErrorInvalidValue;
    if (g.blocked != 1 || g.kg * 16 < g.K || g.pg * 16 < g.P) return hipErrorInvalidValue;
    if (!wino_fused_available(g.n, g.k)) return hipErrorInvalidValue;
    if (config == 1 && !wino_fused_has_big_block(g.n, g.k)) return hipErrorInvalidValue;
    if (config != 1) return dispatch_fused(g, 0, AT, Ub, Vb, bias, y, s, FusedRange{});
    int p_big = 0;
    const hipError_t eq = big_block_share(g, &p_big);
    if (eq != hipSuccess) return eq;
    const int pblocks = (g.P + 63) / 64;
    hipError_t e = dispatch_fused(g, 1, AT, Ub, Vb, bias, y, s, FusedRange{0, p_big, nullptr});
    if (e != hipSuccess || p_big == pblocks) return e;
    return dispatch_fused(g, 0, AT, Ub, Vb, bias, y, s, FusedRange{2 * p_big, -1, nullptr});
}

// kernels one call of launch_wino_fused enqueues (1, or 2 when the tail of the tiles goes to 32 x 32 workgroups)
int wino_fused_launch_count(const WinoGeom& g, int config)
{
    if (config != 1 || !wino_fused_has_big_block(g.n, g.k)) return 1;
    int p_big = 0;
    if (big_block_share(g, &p_big) != hipSuccess) { (void)hipGetLastError(); return 1; }
    const int pblocks = (g.P + 63) / 64;
    return (p_big > 0 && p_big < pblocks) ? 2 : 1;
}

}  // namespace mnnconv
