// Launch functions of the gfx950 kernels.  Raw device pointers and a hipStream_t;
// every launcher validates what its kernel assumes and returns hipError_t.
#pragma once
#include <hip/hip_runtime_api.h>
#include <cstdint>

namespace mnnconv {

constexpr int kMaxAlphaT = 12;   // largest alpha = n + k - 1 the transform kernels are built for

// Transform matrix handed to kernels by value (lands in SGPRs).
template <int R, int C>
struct MatArg { float v[R][C]; };

struct WinoGeom {
    int N, C, H, W, K;          // input x[N][C][H][W], K output channels
    int Ho, Wo;                 // output plane
    int pad_h, pad_w;
    int n, k, alpha;            // F(n, k), alpha = n + k - 1
    int th, tw;                 // tiles per image: ceil(Ho/n), ceil(Wo/n)
    int P;                      // N * th * tw
    int ldp;                    // row length of V / M rows (P rounded up to 4)
    int ldk;                    // row length of U rows (K rounded up to 4)
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
};
hipError_t launch_gemm_f32(const GemmProblem& p, hipStream_t s);

// Wt[r][k] = w[k][r], r < R = C*kh*kw, row length ldk (zero padded)
hipError_t launch_weight_transpose(const float* w, float* Wt, int K, int R, int ldk, hipStream_t s);

struct DirectGeom {
    int N, C, H, W, K, kh, kw, Ho, Wo;
    int stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
};
// Sliding-window convolution straight from the definition.
hipError_t launch_direct_conv(const DirectGeom& g, const float* x, const float* w, const float* bias,
                              float* y, hipStream_t s);

}  // namespace mnnconv
