/*
 * mnn_conv.h -- C ABI of the MI355X (gfx950) convolution library.
 *
 * The library implements the data-parallel hot path of the MNN paper
 * (arXiv 2002.12418):
 *   - pre-inference scheme selection per layer shape        (Section 3.2)
 *   - Winograd convolution F(n x n, k x k) with generated
 *     transform matrices; kernels that are not square with
 *     one matrix set per axis: 1 x k, k x 1 as F(1 x n, 1 x k) /
 *     F(n x 1, k x 1), k_h x k_w as F(n x n, k_h x k_w)      (Section 3.3.1)
 *   - k = 1 convolution as one large matrix multiplication  (Sections 3.2 (1), 3.3.2)
 *   - sliding-window (direct) convolution as the fallback   (Section 3.2 (1))
 *
 * Conventions
 *   - Every function returns MNN_OK (0) or a negative mnn_status; nothing is
 *     thrown across the boundary.  mnn_last_error() gives a thread-local
 *     message for the last failure on the calling thread.
 *   - "device" pointers are HIP device addresses on the current device,
 *     "host" pointers are ordinary process memory.  Tensors are float32,
 *     dense, NCHW (input x[N][C][H][W], output y[N][K][H_o][W_o]) and KCRS
 *     (weight w[K][C][kh][kw]); groups = 1.
 *   - H_o = floor((H + 2*pad_h - dil_h*(kh-1) - 1)/stride_h) + 1, W_o alike;
 *     the operation is a cross-correlation with zero padding plus bias.
 *   - Streams are hipStream_t passed as void* (NULL = the default stream).
 *   - A plan owns its workspace; mnn_conv_run allocates nothing and never
 *     synchronises the host (preparation-execution decoupling, Section 3.2).
 *   - Threading: plan, chain and Strassen handles are not thread-safe.  The calls that run a handle
 *     (mnn_conv_run, _run_stage, _run_timed, _set_weights, mnn_chain_run / _replay, mnn_strassen_run) share its
 *     workspace (V, M, the split-K slices), so one handle serves one stream at a time: work enqueued through it
 *     on a second stream, or from a second thread, while earlier work is still running races on that workspace.
 *     Different handles are independent; the process-wide caches are guarded by locks.
 */
#ifndef MNN_CONV_H
#define MNN_CONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MNN_OK = 0,
    MNN_E_INVALID_ARG = -1,   /* NULL pointer, non-positive size, empty output ...        */
    MNN_E_UNSUPPORTED = -2,   /* valid request the library does not implement             */
    MNN_E_HIP = -3,           /* a HIP runtime call failed (message holds hipGetErrorString) */
    MNN_E_OOM = -4,           /* device allocation failed                                 */
    MNN_E_NO_DEVICE = -5      /* no usable GPU in this process                            */
} mnn_status;

/* Layer shape: x[n][c_in][h][w] (*) w[c_out][c_in][kh][kw]. */
typedef struct { int32_t n, c_in, h, w, c_out, kh, kw; } mnn_conv_shape;
typedef struct { int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w; } mnn_conv_geom;

/* The scheme pool of Section 3.2 (1). */
typedef enum {
    MNN_SCHEME_AUTO = 0,      /* let the planner decide (only meaningful in options)      */
    MNN_SCHEME_DIRECT = 1,    /* sliding window                                           */
    MNN_SCHEME_WINOGRAD = 2,  /* F(tile_n x tile_n, k x k)                                */
    MNN_SCHEME_GEMM1X1 = 3    /* k = 1, stride 1, pad 0: one matrix multiplication        */
} mnn_scheme_kind;

/* Operand precision of the matrix-multiplication stage (accumulation is always fp32). */
typedef enum {
    MNN_GEMM_FP32 = 0,        /* fp32 operands, v_mfma_f32_32x32x2_f32                    */
    MNN_GEMM_BF16 = 1,        /* operands rounded to bf16 (RNE), v_mfma_f32_32x32x16_bf16 */
    MNN_GEMM_BF16X3 = 2       /* each operand split into bf16 hi + lo, product = hi*hi + hi*lo + lo*hi on
                                 the bf16 matrix cores: about 16 mantissa bits, fp32-grade results    */
} mnn_gemm_prec;

typedef struct {
    int32_t kind;             /* mnn_scheme_kind                                          */
    int32_t tile_n;           /* n of F(n,k); 0 unless kind == MNN_SCHEME_WINOGRAD        */
    int32_t prec;             /* mnn_gemm_prec                                            */
    int32_t variant;          /* kernel arrangement of the scheme, see MNN_WINO_*; 0 otherwise */
    float   est_ms;           /* time measured by the planner; < 0 when it was not timed  */
} mnn_scheme;

/* Kernel arrangements of a Winograd scheme (all compute the same F(n,k)).  For MNN_SCHEME_GEMM1X1 the variant
 * field of mnn_scheme (and force_variant) is the number of Strassen levels, 0..2 (Section 3.3.2). */
enum {
    MNN_WINO_UNFUSED = 0,     /* input transform, batched GEMM writing M, output transform        */
    MNN_WINO_FUSED_OUT_32 = 1,/* input transform, GEMM with the output transform in its epilogue,
                                 32 channels x 32 tiles per workgroup; M is never stored           */
    MNN_WINO_FUSED_OUT_64 = 2,/* the same with 64 channels x 64 tiles per workgroup of 8 wavefronts
                                 (where the registers of two wavefronts per SIMD allow it)         */
    MNN_WINO_VARIANTS = 3
};

typedef struct {
    int32_t force_kind;       /* MNN_SCHEME_AUTO or the scheme to use without timing      */
    int32_t force_tile_n;     /* with force_kind == WINOGRAD: the n to use (0 = analytic) */
    int32_t force_prec;       /* mnn_gemm_prec used for forced schemes                    */
    int32_t force_variant;    /* MNN_WINO_* used for a forced Winograd scheme; -1 = time the variants */
    int32_t allow_bf16;       /* 1: AUTO may also time bf16-matrix-core candidates: BF16X3 for every scheme with a
                                 separate GEMM stage, plain BF16 for the 1x1 and sliding-window schemes only
                                 (plain bf16 Winograd operands miss the 2e-2 bound for most tiles)   */
    int32_t alpha_max;        /* largest n + k - 1 the planner may generate (default and maximum 10:
                                 beyond that the fp32 error of the transforms exceeds 1e-3)          */
    float   point_scale_f;    /* f of the Winograd generator (Section 3.3.1).  0 (default): the paper's 0.5 up to
                                 alpha = 8 and 0.425 for alpha = 9 and 10, where 0.5 no longer gives the least fp32
                                 error; > 0: that f for every tile */
    int32_t plan_warmup;      /* untimed launches per candidate (default 2)               */
    int32_t plan_iters;       /* timed launches per candidate (default 10)                */
    int32_t use_cache;        /* 1 (default): consult / fill the process-wide choice cache */
    float   prune_ratio;      /* > 1: candidates whose predicted time (mnn_conv_predict_ms) exceeds prune_ratio times
                                 the best predicted one are not timed; 0 (default): time every candidate */
} mnn_conv_options;

typedef struct mnn_conv_plan_s* mnn_conv_plan_t;

/* Stages of a plan, for per-stage timing and inspection. */
enum {
    MNN_STAGE_FILTER = 0,     /* weight preparation: G w G^T (Winograd) or transposition  */
    MNN_STAGE_INPUT = 1,      /* B^T d B over all tiles                                   */
    MNN_STAGE_GEMM = 2,       /* matrix multiplication (or the whole direct / 1x1 kernel) */
    MNN_STAGE_OUTPUT = 3,     /* A^T m A + bias                                           */
    MNN_STAGE_COUNT = 4
};

/* Plan buffers that tests may look at (device memory owned by the plan). */
enum {
    MNN_BUF_U = 0,            /* prepared weights.  Winograd, unfused: [alpha^2][C][ldk] (ldk = c_out rounded up to 4),
                                 element (xi, c, k) = (G w[k][c] G^T)[xi / alpha][xi % alpha];
                                 fused variants: [b][c/4][a][kg][c%4][k%16], xi = a*alpha + b (kg groups of 16
                                 output channels, channel groups padded to whole 16-channel chunks) */
    MNN_BUF_V = 1,            /* transformed input tiles, unfused: [alpha^2][C][ldp] (ldp = P rounded up to 4), or, when
                                 mnn_plan_info.tiled is set (layers with many tiles), [C][pb][alpha^2][64]: element
                                 (xi, c, p) at ((c*pb + p/64)*alpha^2 + xi)*64 + p%64, ldp = 64*pb;
                                 fused variants: [b][c/4][a][pg][c%4][p%16]                          */
    MNN_BUF_M = 2             /* products [alpha^2][c_out][ldp], or [c_out][pb][alpha^2][64] when tiled (unfused variant only) */
};

typedef struct {
    int32_t alpha, tile_n, tiles_h, tiles_w;  /* Winograd geometry (0 for other schemes)  */
    int32_t p;                /* number of tiles N * tiles_h * tiles_w                    */
    int32_t ldp, ldk;         /* leading dimensions of V/M rows and of U rows             */
    int32_t kg, pg;           /* fused variants: allocated 16-wide groups along c_out and along P */
    int32_t h_out, w_out;
    int32_t alpha_w, tile_n_w; /* kernels that are not square: alpha and tile_n describe the H axis, these the W axis
                                  (alpha = tile_n + k_h - 1, alpha_w = tile_n_w + k_w - 1); an axis with a single tap
                                  has alpha = tile_n = 1; U, V, M hold alpha * alpha_w positions.  Equal to alpha,
                                  tile_n for square kernels. */
    int32_t tiled, pb;         /* tiled != 0: V and M use the [channel][pb][position][64] layout described at MNN_BUF_V,
                                  pb = ceil(p / 64) blocks of 64 tiles */
} mnn_plan_info;

/* Fills *opt with the defaults listed above.  Host. */
int mnn_conv_options_default(mnn_conv_options* opt);

/*
 * Pre-inference for one layer (Section 3.2): validates the shape, enumerates the
 * candidate schemes (k = 1, stride 1, pad 0 -> GEMM; stride or dilation != 1, or more
 * than 7 taps on an axis -> sliding window only; otherwise sliding window and every
 * F(n,k) with n >= 2 and n + k - 1 <= alpha_max, k the long side of the kernel -- at most
 * 8 when the kernel has several taps on both axes and is not square), and unless a scheme is forced
 * or cached, times every candidate on the device with scratch tensors and
 * keeps the fastest (ties: smaller alpha).  Allocates the chosen scheme's
 * workspace.  `stream` is used for the timing launches and is synchronised.
 * shape, geom: host, read only.  options: host or NULL for defaults.
 * *out_plan is set only on success; release it with mnn_conv_plan_destroy.
 */
int mnn_conv_plan(const mnn_conv_shape* shape, const mnn_conv_geom* geom,
                  const mnn_conv_options* options, void* stream, mnn_conv_plan_t* out_plan);

/* The scheme the plan runs: the member of the scheme pool that the cost evaluation of Section 3.2 (1) selected
 * (or the forced one), with the time it measured.  Host. */
int mnn_conv_plan_scheme(mnn_conv_plan_t plan, mnn_scheme* out);

/* The scheme pool of Section 3.2 (1) for this layer -- all schemes the planner considered -- with the cost
 * measured for each (est_ms >= 0; < 0: pruned, did not fit or does not apply).  Writes at most `cap` entries to
 * out (may be NULL with cap 0) and the total to *count.  Host. */
int mnn_conv_plan_candidates(mnn_conv_plan_t plan, mnn_scheme* out, int32_t cap, int32_t* count);

/* Human-readable description of what the plan launches, e.g. "F(4,3) unfused gemm=128x64x16_w2x2".
 * Writes at most cap bytes including the terminating NUL.  Host. */
int mnn_conv_plan_describe(mnn_conv_plan_t plan, char* buf, size_t cap);

/* Geometry of the plan.  Host. */
int mnn_conv_plan_info(mnn_conv_plan_t plan, mnn_plan_info* out);

/* Bytes of device memory the plan owns (workspace + prepared weights): what pre-inference allocated so that
 * inference allocates nothing (preparation-execution decoupling, Section 3.2).  0 for a NULL plan. */
size_t mnn_conv_workspace_bytes(mnn_conv_plan_t plan);

/*
 * Inference for one layer: enqueues the plan's kernels on `stream`.
 * input, weight, bias (may be NULL), output: device, float32, layouts above;
 * input/weight/bias are read only, output is overwritten.  The prepared
 * weights (Winograd: U = G w G^T, Section 3.3.1) are rebuilt only when `weight`
 * differs from the pointer of the previous call or after
 * mnn_conv_invalidate_weights; otherwise the call launches only the
 * per-inference stages.  The library cannot see the CONTENTS of `weight` change:
 * after writing new values to the same address call mnn_conv_set_weights (or
 * mnn_conv_invalidate_weights) before the next run.  Returns MNN_E_HIP if a launch fails.
 */
int mnn_conv_run(mnn_conv_plan_t plan, const float* input, const float* weight,
                 const float* bias, float* output, void* stream);

/*
 * mnn_conv_run for callers that cannot allocate device memory at all: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  One call does what mnn_conv_plan with a forced fp32 scheme followed by
 * mnn_conv_run does -- tile_n >= 2: Winograd F(tile_n, k) with separate transform and GEMM kernels (square
 * kernels and kernels that are not square alike); tile_n == 0: the sliding window, or the 1x1 GEMM for a
 * pointwise layer -- but the prepared weights, V and M live in a fixed array inside the library's code object
 * (mnn_conv_static_scratch_bytes() = 64 MiB per GPU, held until the process ends) instead of a plan's workspace.
 * The call allocates and frees no device memory, synchronises nothing, times nothing (the GEMM tile configuration
 * comes from the shape alone) and prepares the weights on every call.  It enqueues one clearing kernel and the
 * scheme's 2 to 4 kernels on `stream`.
 * shape, geom: host.  input, weight, bias (may be NULL), output: device, float32, layouts above.
 * Errors: MNN_E_INVALID_ARG; MNN_E_UNSUPPORTED when the scheme does not apply to the layer or its scratch
 * memory (prepared weights + V + M, each rounded up to 256 bytes) exceeds the array -- the message names both
 * sizes; MNN_E_HIP.
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap in time (different streams,
 * different threads) race.  Calls on one stream are ordered and safe.
 */
int mnn_conv_run_static(const mnn_conv_shape* shape, const mnn_conv_geom* geom, int32_t tile_n, const float* input,
                        const float* weight, const float* bias, float* output, void* stream);
size_t mnn_conv_static_scratch_bytes(void);

/* Same work as mnn_conv_run repeated `iters` times with HIP events around each
 * stage; synchronises `stream` and writes the mean milliseconds per stage to
 * stage_ms[MNN_STAGE_COUNT] (host; stages the scheme does not have get 0;
 * MNN_STAGE_FILTER is run and timed every iteration here). */
int mnn_conv_run_timed(mnn_conv_plan_t plan, const float* input, const float* weight,
                       const float* bias, float* output, void* stream, int32_t iters,
                       float* stage_ms);

/* Runs a single stage (MNN_STAGE_*) of the plan; the stages before it must have
 * run with the same tensors.  For per-kernel profiling. */
int mnn_conv_run_stage(mnn_conv_plan_t plan, int32_t stage, const float* input, const float* weight,
                       const float* bias, float* output, void* stream);

/* Prepares the weights now: enqueues G w G^T (Section 3.3.1; computed once per weight set, not per inference)
 * or the transposition of the 1x1 / sliding-window schemes on `stream` and remembers `weight` as prepared, so
 * that the following mnn_conv_run calls with this pointer launch only the per-inference stages.  This is the
 * explicit form of what mnn_conv_run does when it sees a new pointer; it is the call to make after the values
 * behind an unchanged pointer were rewritten.  weight: device, float32, KCRS, read only.
 * Errors: MNN_E_INVALID_ARG (NULL), MNN_E_HIP. */
int mnn_conv_set_weights(mnn_conv_plan_t plan, const float* weight, void* stream);

/* Marks the prepared weights (G w G^T of Section 3.3.1, computed once per weight set) as stale: the next
 * mnn_conv_run prepares them again from its `weight` argument.  Host; launches nothing. */
int mnn_conv_invalidate_weights(mnn_conv_plan_t plan);

/* Device address and size in bytes of one of the plan's buffers (MNN_BUF_*);
 * *ptr is NULL when the scheme has no such buffer. */
int mnn_conv_plan_buffer(mnn_conv_plan_t plan, int32_t which, void** ptr, size_t* bytes);

/* Copies one of the plan's buffers to host memory after synchronising `stream` (inspection, tests).
 * dst: host, at least `bytes` bytes; bytes must not exceed the buffer size. */
int mnn_conv_read_buffer(mnn_conv_plan_t plan, int32_t which, void* dst, size_t bytes, void* stream);

/* Ends what pre-inference set up (Section 3.2): frees the plan's workspace and prepared weights.  The choices it
 * left in the process-wide cache stay.  The caller makes sure that no work enqueued through the plan is still
 * running.  NULL is allowed. */
void mnn_conv_plan_destroy(mnn_conv_plan_t plan);

/*
 * Winograd generator (Section 3.3.1 (3)).  Host only.  Interpolation points are
 * 0, +f, -f, +2f, -2f, ... (the first n + k - 2 of them) and infinity.  Writes
 * row-major AT[n][alpha], G[alpha][k], BT[alpha][alpha], alpha = n + k - 1, such
 * that  AT [ (G g) (.) (BT d) ]_i = sum_j d[i+j] g[j].
 */
int mnn_conv_get_transforms(int32_t n, int32_t k, float f, float* AT, float* G, float* BT);

/*
 * Analytic cost of Section 3.2 (1).  Host only.
 * mnn_conv_analytic_cost: cost of the whole output plane with output tile n,
 *   ceil(o_h/n) * ceil(o_w/n) * [2 i_c a^3 + i_c o_c a^2 + n a (2n + k - 1)], a = n + k - 1.
 * mnn_conv_analytic_tile: the n in [1, alpha_max - k + 1] with the least such cost
 *   (1 means sliding window); ties go to the smaller n.
 */
int mnn_conv_analytic_cost(int32_t k, int32_t i_c, int32_t o_c, int32_t o_h, int32_t o_w,
                           int32_t n, double* cost);
int mnn_conv_analytic_tile(int32_t k, int32_t i_c, int32_t o_c, int32_t o_h, int32_t o_w,
                           int32_t alpha_max, int32_t* n_hat);

/*
 * Cost of an operator on this device in the form of Section 3.2 (2): work / FLOPS + t_schedule per kernel,
 * with the memory side added (a kernel takes max(flops / FLOPS, bytes / bandwidth) + t_schedule), summed over
 * the kernels a scheme launches.  The three constants are "known constants for a specific backend"; the
 * defaults were measured on an MI355X (fp32 matrix-core rate of the GEMM, rate of the transform kernels,
 * dispatch-to-dispatch time of dependent kernels); mnn_conv_calibrate re-measures them on `stream` (a large
 * product, a large copy, a chain of empty kernels; about 50 ms) and installs the result process-wide.
 * mnn_conv_predict_ms: host only; the predicted milliseconds of `scheme` for the layer.
 */
typedef struct {
    double flops;             /* fp32 multiply-add rate of the matrix-multiplication stage, FLOP/s */
    double bytes_per_s;       /* sustained HBM rate of a streaming kernel, B/s                     */
    double t_schedule_ms;     /* fixed cost per kernel launch in a dependent chain, ms             */
} mnn_device_model;
int mnn_conv_get_device_model(mnn_device_model* out);
int mnn_conv_set_device_model(const mnn_device_model* model);
int mnn_conv_calibrate(void* stream, mnn_device_model* out);
int mnn_conv_predict_ms(const mnn_conv_shape* shape, const mnn_conv_geom* geom, const mnn_scheme* scheme,
                        double* ms);

/*
 * Upper limits of the two device rates of Section 3.2 (2), measured on `stream` (about 20 ms): the rate at
 * which the GPU issues fp32 matrix-core instructions from registers with no memory access in the loop, and the
 * rate of a plain 16-byte copy kernel over 256 MiB (bytes read plus bytes written per second).  These are the
 * ceilings a roofline fraction can be taken against next to the published figures; the cost model does not
 * use them.  Allocates and frees its own device buffers; synchronises `stream`.  `out` is host memory.
 * Errors: MNN_E_INVALID_ARG (NULL out), MNN_E_NO_DEVICE, MNN_E_OOM, MNN_E_HIP.
 */
typedef struct {
    double mfma_f32_flops;    /* FLOP/s of back-to-back fp32 32x32x2 matrix-core instructions, whole device */
    double copy_bytes_per_s;  /* B/s (read + write) of a streaming copy kernel                              */
} mnn_device_peaks;
int mnn_measure_device_peaks(void* stream, mnn_device_peaks* out);

/* The candidate list mnn_conv_plan would time for this layer, without touching
 * the device.  Host only.  Same cap / count convention as above. */
int mnn_conv_enumerate(const mnn_conv_shape* shape, const mnn_conv_geom* geom,
                       const mnn_conv_options* options, mnn_scheme* out, int32_t cap, int32_t* count);

/* Index of the candidate the planner keeps given measured times (est_ms):
 * the least est_ms; among times within 2 % of it, the smallest alpha, then the
 * fp32 variant.  Candidates with est_ms < 0 are ignored.  Host only. */
int mnn_conv_select(const mnn_scheme* cands, int32_t count, int32_t k, int32_t* chosen);

/*
 * The matrix-multiplication unit on its own (Sections 3.3.1 (2), 3.3.2): for b < batch
 *   D_b[m][col] = sum_{r<R} At_b[r][m] * B_b[r][col]  (+ bias[m] when bias != NULL),  m < M, col < ncols.
 * All pointers are device memory, float32.  At is the left operand stored transposed,
 * At_b = At + b*strideA_batch, row length lda (multiple of 4, >= M, 16-byte aligned base).
 * B element (r, col) lives at  B + b*strideB_batch + (col / L)*strideB_img + r*strideB_row + col % L,
 * D element (m, col) at        D + b*strideD_batch + (col / L)*strideD_img + m*strideD_row + col % L
 * (L = run of columns that is contiguous in memory; strides in elements).
 * prec is a mnn_gemm_prec.  variant 0 picks the tile configuration from the shape;
 * 1..mnn_gemm_variant_count(prec)-1 force one.
 */
typedef struct {
    int32_t M, ncols, R, batch, lda, L, variant, prec;
    int64_t strideA_batch, strideB_batch, strideB_img, strideB_row, strideD_batch, strideD_img, strideD_row;
} mnn_gemm_desc;
int mnn_gemm_f32(const mnn_gemm_desc* desc, const float* At, const float* B, const float* bias, float* D,
                 void* stream);
int mnn_gemm_variant_count(int32_t prec);

/*
 * Strassen's algorithm for one large product (Section 3.3.2), same operand layout as mnn_gemm_f32 with
 * batch = 1 and prec = MNN_GEMM_FP32.  `levels` recursion levels, each: the 4 + 4 additions on the operand
 * quadrants, 7 half-size products, 7 additions on the results (the count the paper gives); level l multiplies
 * 7^l blocks in one batched GEMM.  levels = 0 is the plain GEMM.  levels > 0 needs M and ncols divisible by
 * 4 * 2^levels, R by 2^levels, and L, lda and all strides divisible by 4 (else MNN_E_UNSUPPORTED).
 * mnn_strassen_levels_by_rule (host): how many levels, at most max_levels, the paper's rule allows --
 *   m n k - 7 (m/2)(n/2)(k/2) > 4 (m/2)(k/2) + 4 (n/2)(k/2) + 7 (m/2)(n/2)  for [n,k] x [k,m] at every level --
 *   under those divisibility conditions.
 * mnn_strassen_create allocates all temporaries and times the tile configuration of the leaf GEMM on `stream`.
 * mnn_strassen_set_left expands the left operand At (device, 16-byte aligned; the weights in the convolution
 * use) once; mnn_strassen_run multiplies it with B (device) into D (device, + bias[m] if bias != NULL),
 * enqueuing 2*levels + 1 kernels.  At must stay valid while the handle is used with levels = 0.
 */
typedef struct mnn_strassen_s* mnn_strassen_t;
int mnn_strassen_levels_by_rule(int32_t M, int32_t R, int32_t ncols, int32_t max_levels);
int mnn_strassen_create(const mnn_gemm_desc* desc, int32_t levels, void* stream, mnn_strassen_t* out);
int mnn_strassen_set_left(mnn_strassen_t h, const float* At, void* stream);
int mnn_strassen_run(mnn_strassen_t h, const float* B, const float* bias, float* D, void* stream);
int mnn_strassen_info(mnn_strassen_t h, int32_t* levels, int32_t* launches, size_t* workspace_bytes);
void mnn_strassen_destroy(mnn_strassen_t h);
const char* mnn_gemm_variant_name(int32_t prec, int32_t variant);

/*
 * A chain of convolution layers prepared once and executed many times (Section 3.2,
 * "preparation-execution decoupling", Table 2).  Layer i+1 consumes what layer i
 * produces: its n, c_in, h, w must equal layer i's n, c_out, h_out, w_out.
 *
 * mnn_chain_create does all preparation: plans every layer as mnn_conv_plan does
 * (same options, same caches), walks the chain once without running it to learn
 * when each buffer is first and last needed (activation i: layers i and i+1; the
 * Winograd-domain workspace of layer i: layer i only), places all of them in ONE
 * device allocation with lifetime-based reuse, and allocates the prepared weights.
 * After it returns, no call below allocates or frees device memory.
 *
 * mnn_chain_set_weights prepares layer i's weights (device, float32, KCRS; bias
 * device or NULL) on `stream`; the chain keeps U / the transposed weights and a
 * copy of the bias, the caller's buffers may be released once `stream` has run.
 *
 * mnn_chain_run enqueues every kernel of every layer on `stream` (input: layer 0's
 * NCHW tensor, output: the last layer's; both device, caller-owned).
 * mnn_chain_capture records the same launches for fixed input/output addresses
 * into a HIP graph (on a stream the chain owns; nothing executes), and
 * mnn_chain_replay launches that graph on `stream` -- the analogue of a
 * pre-recorded command buffer.  A chain must not run on two streams at once.
 * Errors: MNN_E_INVALID_ARG (shapes that do not connect, NULL pointers, weights
 * not set, replay without capture), MNN_E_HIP, MNN_E_OOM, MNN_E_NO_DEVICE.
 */
typedef struct mnn_chain_s* mnn_chain_t;
typedef struct {
    mnn_conv_shape shape;
    mnn_conv_geom geom;
} mnn_chain_layer;
typedef struct {
    int32_t n_layers;
    int32_t kernels_per_run;     /* launches of one mnn_chain_run */
    int32_t graph_nodes;         /* nodes of the captured graph, 0 before mnn_chain_capture */
    int32_t reserved;
    uint64_t arena_bytes;        /* the one allocation: activations + workspaces with reuse */
    uint64_t unshared_bytes;     /* the same buffers without reuse (sum of their sizes) */
    uint64_t live_peak_bytes;    /* most bytes alive at any layer: lower bound for arena_bytes */
    uint64_t weight_bytes;       /* prepared weights and bias copies */
} mnn_chain_info_t;

int mnn_chain_create(const mnn_chain_layer* layers, int32_t n_layers, const mnn_conv_options* options,
                     void* stream, mnn_chain_t* out_chain);
int mnn_chain_set_weights(mnn_chain_t chain, int32_t layer, const float* weight, const float* bias, void* stream);
int mnn_chain_run(mnn_chain_t chain, const float* input, float* output, void* stream);
int mnn_chain_capture(mnn_chain_t chain, const float* input, float* output);
int mnn_chain_replay(mnn_chain_t chain, void* stream);
int mnn_chain_info(mnn_chain_t chain, mnn_chain_info_t* out);
int mnn_chain_layer_scheme(mnn_chain_t chain, int32_t layer, mnn_scheme* out);
int mnn_chain_layer_describe(mnn_chain_t chain, int32_t layer, char* buf, size_t cap);
/* Copies intermediate activation `layer` (the output of that layer, layer < n_layers-1) to host memory
 * after synchronising `stream`; valid only until the next run overwrites it.  For tests. */
int mnn_chain_read_activation(mnn_chain_t chain, int32_t layer, float* dst, size_t bytes, void* stream);
void mnn_chain_destroy(mnn_chain_t chain);

/*
 * The pool planner on its own.  Host only.  Buffer i has bytes[i] >= 0 bytes and is
 * alive from operator first[i] to operator last[i] inclusive.  Writes offsets[i]
 * (multiples of align, a power of two) such that buffers alive at the same time
 * never overlap, and the pool size to *total.
 */
int mnn_arena_plan(const int64_t* bytes, const int32_t* first, const int32_t* last, int32_t count,
                   int64_t align, int64_t* offsets, int64_t* total);

/* Process-wide cache of planner choices keyed by device, shape, geometry and options. */
int mnn_conv_cache_size(void);
void mnn_conv_cache_clear(void);

/* Pre-inference results outlive the process: mnn_conv_cache_save writes every cached choice (scheme per
 * layer shape, GEMM tile configuration per matrix shape) to a text file, mnn_conv_cache_load merges such a
 * file into the cache, so that a later mnn_conv_plan for a known shape launches no timing kernels.
 * path: host, NUL-terminated.  Entries are keyed by the HIP device ordinal they were measured on. */
int mnn_conv_cache_save(const char* path);
int mnn_conv_cache_load(const char* path);

/* Message of the last failure on the calling thread (empty string if none).  Host. */
const char* mnn_last_error(void);
/* 100 * major + minor of this ABI; plan-cache files carry their own format number. */
int mnn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MNN_CONV_H */
