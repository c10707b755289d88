// Launch functions of the gfx950 kernels.  Raw device pointers and a hipStream_t;
// every launcher validates what its kernel assumes and returns hipError_t.
#pragma once
#include <hip/hip_runtime_api.h>
#include <cstddef>
#include <cstdint>

namespace mnnconv {

// Largest alpha = n + k - 1 the Winograd kernels are built for.  In fp32 the error of the generated
// transforms grows quickly with alpha: about 3e-4 of the output range at alpha = 10 and above 1e-2 from
// alpha = 11 on, which is outside the accuracy this library promises.
constexpr int kMaxAlphaT = 10;

// Transform matrix handed to kernels by value (lands in SGPRs).
template <int R, int C>
struct MatArg { float v[R][C]; };

struct WinoGeom {
    int N, C, H, W, K;          // input x[N][C][H][W], K output channels
    int Ho, Wo;                 // output plane
    int pad_h, pad_w;
    int n, k, alpha;            // F(n, k), alpha = n + k - 1 (along H when the kernel is not square)
    int nw, kw, alpha_w;        // the same along W; equal to n, k, alpha for square kernels.  An axis along
                                // which the kernel has one tap is left untransformed: n = k = alpha = 1.
    int th, tw;                 // tiles per image: ceil(Ho/n), ceil(Wo/nw)
    int P;                      // N * th * tw
    int ldp;                    // row length of V / M rows (P rounded up to 4)
    int ldk;                    // row length of U rows (K rounded up to 4)
    // Blocked ("MFMA-native") layout used by the fused kernel instead of the row layouts
    // (xi = a*alpha + b):  Ub[b][c/4][a][k/16][c%4][k%16],  Vb[b][c/4][a][p/16][c%4][p%16]
    int blocked;                // 0: row layouts U[xi][c][ldk], V[xi][c][ldp];  1: blocked
    int kg, pg;                 // allocated 16-column groups along K and along P
    int cchunks;                // allocated 4-channel groups (>= ceil(C/4), padded to whole chunks)
    // Tiled row layout (blocked == 0, tiled == 1): V[c][p/64][xi][p%64], M[k][p/64][xi][p%64] -- the alpha^2 values of 64
    // consecutive tiles of one channel are one contiguous run, which is exactly what one wavefront of the transform kernels
    // writes or reads; ldp = 64 * pb.
    int tiled;
    int pb;                     // 64-tile blocks: ceil(P / 64)
    int itx_waves;              // input transform: resident wavefronts per CU to allow (10, 12, 16 or 20), 0 = as many as fit
};

// U[xi][c][k] = (G w[k][c] G^T)[xi/alpha][xi%alpha]          (Section 3.3.1, G W G^T)
hipError_t launch_filter_transform(const WinoGeom& g, const float* G /*host, alpha x k*/,
                                   const float* w, float* U, hipStream_t s);

// V[xi][c][p] = (B^T d B)[xi/alpha][xi%alpha], d = input tile p of channel c   (B^T X B)
hipError_t launch_input_transform(const WinoGeom& g, const float* BT /*host, alpha x alpha*/,
                                  const float* x, float* V, hipStream_t s);

// y[img][k][ty*n+i][tx*n+j] = (A^T m A)[i][j] + bias[k], m[a][b] = M[a*alpha+b][k][p]   (A^T [.] A)
hipError_t launch_output_transform(const WinoGeom& g, const float* AT /*host, n x alpha*/,
                                   const float* M, const float* bias, float* y, hipStream_t s);

bool winograd_kernels_available(int n, int k);

// One-dimensional Winograd for kernels with a single row or column (1 x k, k x 1; Section 3.3.1: "kernels of
// any size"): F(n, k) along the long axis, identity along the other.  Row layouts only (g.blocked == 0):
// U[(i*alpha_w + j)][c][ldk], V and M likewise.  Matrices of the untransformed axis are the 1 x 1 identity.
bool winograd_rect_kernels_available(int nh, int kh, int nw, int kw);
hipError_t launch_filter_transform_rect(const WinoGeom& g, const float* Gh, const float* Gw, const float* w, float* U,
                                        hipStream_t s);
hipError_t launch_input_transform_rect(const WinoGeom& g, const float* BTh, const float* BTw, const float* x, float* V,
                                       hipStream_t s);
hipError_t launch_output_transform_rect(const WinoGeom& g, const float* ATh, const float* ATw, const float* M,
                                        const float* bias, float* y, hipStream_t s);

// Winograd-domain product with the inverse transform and bias fused in:
// y = A^T [ sum_c U (.) V ] A + bias, operands in the blocked layout.  M is never stored.
// config 0: 32 channels x 32 tiles per workgroup; config 1: 64 x 64 (only where wino_fused_has_big_block), with the
// tiles of a mostly empty last round of workgroups handed to 32 x 32 workgroups (up to two launches).
bool wino_fused_available(int n, int k);
bool wino_fused_has_big_block(int n, int k);
hipError_t launch_wino_fused(const WinoGeom& g, int config, const float* AT /*host*/, const float* Ub,
                             const float* Vb, const float* bias, float* y, hipStream_t s);
int wino_fused_launch_count(const WinoGeom& g, int config);      // kernels one such call enqueues

// Batched GEMM  D_b[m][col] = sum_r At_b[r][m] * B_b[r][col] (+ bias[m]).
//   At: [batch][R][lda]  (A stored transposed, m contiguous; lda % 4 == 0, 16-byte aligned)
//   B : element (r, col) at  B + b*strideB_batch + (col / L)*strideB_img + r*strideB_row + (col % L)
//   D : element (m, col) at  D + b*strideD_batch + (col / L)*strideD_img + m*strideD_row + (col % L)
// L is the number of consecutive columns that are contiguous in memory (the whole
// row for the Winograd-domain product, H*W for the 1x1 convolution of one image).
struct GemmProblem {
    const float* At; const float* B; float* D; const float* bias;
    int M, Ncols, R, batch;
    int lda;
    int L;
    long long strideA_batch;
    long long strideB_batch, strideB_img, strideB_row;
    long long strideD_batch, strideD_img, strideD_row;
    int variant;                // 0 = choose from the shape; > 0 = a specific tile configuration (tuning, tests)
    int prec;                   // 0: fp32 MFMA; 1: bf16 operands; 2: bf16x3 (hi/lo split, three bf16 MFMAs per product)
    // Split-K (register-staged kernels only): splitk > 1 cuts the reduction of every tile into that many
    // workgroups, which write partial results to splitk_partial (gemm_splitk_workspace floats, 16-byte
    // aligned); a second kernel adds them up in slice order.  0 or 1 = off.
    int splitk;
    float* splitk_partial;
    // Implicit-GEMM gather for the sliding-window scheme (gather != 0): B is the input tensor x[N][C][H][W],
    // row r = (c, kr, ks), column = (img, oy, ox), element = x[img][c][oy*sh - ph + kr*dh][ox*sw - pw + ks*dw] or 0.
    // L must be H_o*W_o; the strideB_* fields are ignored.
    int gather;
    int cv_C, cv_H, cv_W, cv_kh, cv_kw, cv_sh, cv_sw, cv_ph, cv_pw, cv_dh, cv_dw, cv_Wo;
};
hipError_t launch_gemm_f32(const GemmProblem& p, hipStream_t s);
int gemm_f32_variant_count();
const char* gemm_f32_variant_name(int variant);
// Tile shape of a variant of precision `prec` (false for variants that cannot split K) and the scratch a
// split-K launch needs: floats of partial sums and number of tile counters.
bool gemm_variant_tile(int prec, int variant, int* bm, int* bn, int* bk);
inline int gemm_splitk_ldc(const GemmProblem& p) { return (p.Ncols + 3) / 4 * 4; }    // row length of the partial results
long long gemm_splitk_workspace(const GemmProblem& p, int splitk);                    // floats
hipError_t launch_splitk_reduce(const GemmProblem& p, hipStream_t s);
// bf16 / bf16x3 operand kernels (gemm_bf16.hip); launch_gemm_f32 forwards to them when prec != 0
int gemm_bf16_variant_count();
const char* gemm_bf16_variant_name(int variant);
hipError_t launch_gemm_bf16(const GemmProblem& p, hipStream_t s);
bool gemm_bf16_variant_tile(int variant, int* bm, int* bn, int* bk);
// variants of the table that serves precision `prec`
inline int gemm_variant_count(int prec) { return prec == 0 ? gemm_f32_variant_count() : gemm_bf16_variant_count(); }
inline const char* gemm_variant_name(int prec, int v) { return prec == 0 ? gemm_f32_variant_name(v) : gemm_bf16_variant_name(v); }

// Strassen's algorithm (Section 3.3.2), one level = expand both operands, one batched GEMM, combine.
// A view addresses element (r, c) of a row-major operand at  (c / L) * sImg + r * sRow + c % L  (the column
// mapping of the GEMM: L consecutive columns are contiguous, the next L belong to the next image).
// All of L, sImg, sRow and the half widths must be multiples of 4, bases 16-byte aligned.
struct StrassenView { int L; long long sImg, sRow; };
// src: nb operands [2*rows_half][2*cols_half] (batch stride in floats) -> dst [7*nb][rows_half][cols_half] dense.
// left: the operand is A stored transposed (At[r][m]); otherwise it is B.
hipError_t launch_strassen_expand(bool left, const StrassenView& v, const float* src, long long src_batch_stride, int rows_half,
                                  int cols_half, int nb, float* dst, hipStream_t s);
// src: [7*nb][rows_half][cols_half] dense products -> dst: nb results [2*rows_half][2*cols_half] (+ bias per row, nb = 1).
hipError_t launch_strassen_combine(const StrassenView& v, const float* src, int rows_half, int cols_half, int nb, float* dst,
                                   long long dst_batch_stride, const float* bias, hipStream_t s);

// Wt[r][k] = w[k][r], r < R = C*kh*kw, row length ldk (zero padded)
hipError_t launch_weight_transpose(const float* w, float* Wt, int K, int R, int ldk, hipStream_t s);

// Seeded pseudo-random floats in [lo, hi] (scratch tensors of the timing planner) and zeros written by a kernel
// (dst 16-byte aligned), for memory that code under graph capture has to clear.
hipError_t launch_fill_pattern(float* dst, size_t n_floats, unsigned seed, float lo, float hi, hipStream_t s);
hipError_t launch_fill_zero(float* dst, size_t n_floats, hipStream_t s);

// Device address, on the current device, of the library's fixed scratch array of kStaticScratchBytes bytes (256-byte
// aligned; part of the code object, never allocated or freed; every device holds its own copy, which keeps the contents
// of the last call).  Looks the address up on the first call per device; allocates nothing.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
hipError_t static_scratch(float** ptr);

// Device-rate probes: `workgroups` x 4 waves each issuing 4*iters fp32 32x32x2 matrix-core instructions
// (out: workgroups*256 floats), and a 16-byte-per-lane copy of n_floats (multiple of 4, 16-byte aligned).
hipError_t launch_mfma_issue(float* out, int workgroups, int iters, hipStream_t s);
hipError_t launch_stream_copy(const float* src, float* dst, size_t n_floats, hipStream_t s);

}  // namespace mnnconv
