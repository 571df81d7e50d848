/*
 * jetfire.h -- C ABI of the MI355X (gfx950) per-block INT8 data-flow library.
 *
 * The library implements the hot path of arxiv 2403.12422 ("Jetfire"):
 * tensors are INT8 codes plus one FP32 scale per square BxB block (Sec. 4,
 * Eq. 1), the three matrix products of a linear layer run as INT8 MFMA GEMMs
 * with the block scales folded into an FP32 accumulator and the output
 * re-quantized inside the kernel (Sec. 5, Alg. 1), and GELU / LayerNorm read
 * and write the same format (Sec. 6, Alg. 2, App. A).
 *
 * Conventions for every entry point
 * ---------------------------------
 *  - Every tensor argument is a DEVICE pointer owned by the caller.  The
 *    library never allocates, frees or keeps a pointer after the call returns.
 *  - INT8 code matrices are row-major; unless an explicit leading dimension
 *    is given they are dense (leading dimension = number of columns).  Codes
 *    lie in [-127, 127].
 *  - A scale grid is a dense row-major FP32 matrix (rows/block) x (cols/block).
 *  - `block` is the quantization block size B and must be 32, 64 or 128; every
 *    matrix dimension must be a positive multiple of it, at most 2^24, and a
 *    matrix may hold at most 2^40 elements (JF_ERR_SHAPE otherwise).
 *  - All pointers must be 16-byte aligned (FP32 vectors: 4-byte) and leading
 *    dimensions multiples of 16 elements.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls validate their arguments synchronously, then enqueue kernels on the
 *    stream and return without waiting for them.
 *  - `ws` / `ws_bytes`: caller-provided scratch of at least
 *    jf_workspace_bytes(...) bytes (may be NULL when that is 0).
 *  - Return value: JF_OK or one of the JF_ERR_* codes below; no entry point
 *    throws or aborts.  On JF_ERR_LAUNCH, jf_last_hip_error() returns the HIP
 *    error code of the failed call.  Nothing is launched when an error other
 *    than JF_ERR_LAUNCH is returned.
 *  - Inputs are assumed finite; NaN/Inf inputs and codes of -128 give
 *    unspecified results (never out-of-bounds accesses).
 *
 * Quantizer used by every output (Eq. 1; scale = block max-abs / 127 as one
 * FP32 division, round-half-to-even, all-zero block -> scale 0 and codes 0).
 */
#ifndef JETFIRE_H_
#define JETFIRE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  JF_OK = 0,
  JF_ERR_NULL = 1,      /* a required pointer is NULL */
  JF_ERR_SHAPE = 2,     /* a dimension is <= 0, too large, or not a multiple of block */
  JF_ERR_BLOCK = 3,     /* block is not 32, 64 or 128 */
  JF_ERR_ALIGN = 4,     /* a pointer or leading dimension is misaligned */
  JF_ERR_WORKSPACE = 5, /* ws is NULL or ws_bytes too small */
  JF_ERR_LAUNCH = 6,    /* a HIP call failed; see jf_last_hip_error() */
  JF_ERR_DTYPE = 7      /* unknown x_dtype */
};

/* Operation selectors for jf_workspace_bytes. */
enum {
  JF_OP_QUANTIZE = 0,
  JF_OP_LINEAR_FWD = 1,
  JF_OP_LINEAR_DGRAD = 2,
  JF_OP_LINEAR_WGRAD = 3,
  JF_OP_GELU = 4,
  JF_OP_GELU_BWD = 5,
  JF_OP_LAYERNORM = 6,
  JF_OP_LAYERNORM_BWD = 7
};

/* HIP error code of the most recent failed HIP call made by this library in
 * the calling thread (0 if none). */
int32_t jf_last_hip_error(void);

/* Static, human-readable name of a JF_* code. */
const char* jf_error_string(int32_t code);

/* Scratch bytes an operation needs for the given problem (N tokens, C
 * in-features, D out-features; element-wise ops use N x C and ignore D). */
size_t jf_workspace_bytes(int32_t op, int64_t N, int64_t C, int64_t D, int32_t block);

/*
 * Per-block quantizer Q (Sec. 4, Eq. 1).
 *   x       rows x cols source, FP32 (x_dtype 0) or FP16 (x_dtype 1), row-major,
 *           leading dimension ldx elements.
 *   q, s    out: INT8 codes rows x cols (leading dimension ldq) and the
 *           (rows/block) x (cols/block) scale grid.
 *   qT, sT  optional out (both NULL or both non-NULL): the transposed tensor,
 *           codes cols x rows (leading dimension ldqT) and grid
 *           (cols/block) x (rows/block); equal to quantizing the transposed
 *           source because blocks are square.
 */
int32_t jf_quantize_block(const void* x, int32_t x_dtype, int64_t rows, int64_t cols, int64_t ldx, int32_t block,
                          int8_t* q, int64_t ldq, float* s, int8_t* qT, int64_t ldqT, float* sT, void* stream);

/*
 * Dequantizer Q^-1 of Sec. 4, Eq. 1: out = code * scale, the hand-over from
 * the INT8 data flow to a floating-point operator (Sec. 7.1 keeps multi-head
 * attention in FP16).  q rows x cols codes (dense), s scale grid;
 * out rows x cols with leading dimension ldo (elements), out_dtype 0 = FP32,
 * 1 = FP16 (the FP32 product rounded to nearest even).
 */
int32_t jf_dequantize_block(const int8_t* q, const float* s, int64_t rows, int64_t cols, int32_t block, void* out,
                            int32_t out_dtype, int64_t ldo, void* stream);

/*
 * INT8 linear layer, forward product Y = X W^T (Sec. 4; Sec. 5 Eq. 2; Alg. 1).
 *   X  N x C codes, SX (N/B) x (C/B);  W  D x C codes, SW (D/B) x (C/B).
 *   Y  out N x D codes, SY out (N/B) x (D/B).
 *   Y_f32  optional out (NULL to skip): the N x D FP32 accumulator of Alg. 1
 *          before it is quantized.
 * For each output block the K-blocks are visited in ascending order and
 *   acc = fma(fl32(SX[p,k] * SW[q,k]), (float)(INT32 block product), acc).
 */
int32_t jf_linear_fwd(const int8_t* X, const float* SX, const int8_t* W, const float* SW, int64_t N, int64_t C,
                      int64_t D, int32_t block, int8_t* Y, float* SY, float* Y_f32, void* ws, size_t ws_bytes,
                      void* stream);

/*
 * Input gradient dX = dY W (Sec. 4).  dY N x D, W D x C (the forward's
 * operand, read transposed inside the kernel; its scale grid is reused with
 * swapped indices because blocks are square).  dX out N x C, SdX (N/B) x (C/B).
 */
int32_t jf_linear_dgrad(const int8_t* dY, const float* SdY, const int8_t* W, const float* SW, int64_t N, int64_t C,
                        int64_t D, int32_t block, int8_t* dX, float* SdX, float* dX_f32, void* ws, size_t ws_bytes,
                        void* stream);

/*
 * Weight gradient dW = dY^T X (Sec. 4), contraction over the N tokens.
 * dY N x D, X N x C, both read transposed inside the kernel.
 * Outputs: dW D x C codes + SdW (D/B) x (C/B) (both NULL or both non-NULL)
 * and/or dW_f32 (D x C FP32 accumulator).  At least one output is required.
 */
int32_t jf_linear_wgrad(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX, int64_t N, int64_t C,
                        int64_t D, int32_t block, int8_t* dW, float* SdW, float* dW_f32, void* ws, size_t ws_bytes,
                        void* stream);

/*
 * Both backward products of a layer in one call (Sec. 4): dX = dY W exactly
 * as jf_linear_dgrad and dW = dY^T X exactly as jf_linear_wgrad, same
 * arguments, same results bit for bit.  The two products need the same dY
 * and nothing of each other; for layers whose products are too small to fill
 * the chip one by one (block 32, outputs of a few hundred 64 x 64 tiles) they
 * run as ONE kernel launch, otherwise as two.
 */
int32_t jf_linear_bwd(const int8_t* dY, const float* SdY, const int8_t* W, const float* SW, const int8_t* X,
                      const float* SX, int64_t N, int64_t C, int64_t D, int32_t block, int8_t* dX, float* SdX,
                      float* dX_f32, int8_t* dW, float* SdW, float* dW_f32, void* ws, size_t ws_bytes, void* stream);

/*
 * INT8 GELU (Sec. 6, Alg. 2; App. A: GELU(x) = x Phi(x), exact-erf form).
 * X N x C codes + SX  ->  Y N x C codes + SY.
 */
int32_t jf_gelu_q(const int8_t* X, const float* SX, int64_t N, int64_t C, int32_t block, int8_t* Y, float* SY,
                  void* stream);

/*
 * INT8 GELU backward (App. A): dX = dY * (x phi(x) + Phi(x)), x = the
 * forward's INT8 input.
 */
int32_t jf_gelu_q_bwd(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX, int64_t N, int64_t C,
                      int32_t block, int8_t* dX, float* SdX, void* stream);

/*
 * INT8 LayerNorm (App. A; Alg. 2).  Row statistics (mean, biased variance)
 * are those of the dequantized input; y = (x - mean) * rstd * gamma + beta.
 * gamma, beta: FP32 [C] (Sec. 7.1 keeps them in floating point).
 * Outputs: Y codes + SY, and mean[N], rstd[N] (FP32, saved for backward).
 * Rows may be of any width (no workgroup holds a whole row).
 */
int32_t jf_layernorm_q(const int8_t* X, const float* SX, const float* gamma, const float* beta, float eps, int64_t N,
                       int64_t C, int32_t block, int8_t* Y, float* SY, float* mean, float* rstd, void* stream);

/*
 * INT8 LayerNorm that takes its row statistics from the partials of the
 * preceding Add (App. A, LayerNorm paragraph) instead of a pass over X:
 *   mean_i = (1/L_C) sum_j row_mean[j][i],  E[x^2]_i = (1/C) sum_j row_sumsq[j][i],
 *   var_i = max(E[x^2]_i - mean_i^2, 0),  rstd_i = 1/sqrt(var_i + eps),
 * then y = (x - mean) * rstd * gamma + beta on the dequantized X as above.
 * row_mean, row_sumsq: FP32 (C/block) x N, as written by jf_add_q.
 */
int32_t jf_layernorm_q_partials(const int8_t* X, const float* SX, const float* row_mean, const float* row_sumsq,
                                const float* gamma, const float* beta, float eps, int64_t N, int64_t C, int32_t block,
                                int8_t* Y, float* SY, float* mean, float* rstd, void* stream);

/*
 * INT8 Add (App. A): Y = Q(X1 + X2) on the dequantized operands, the residual
 * connection forward and dx = df(y) + dy backward.  X1, X2: N x C codes with
 * grids S1, S2; Y, SY out.  row_mean / row_sumsq (both NULL or both non-NULL)
 * receive, for every row and block column, the mean and the sum of squares of
 * the FP32 sum over the block's columns -- the row partials that App. A
 * attaches to this operator for the LayerNorm after it.  They are FP32
 * matrices of (C/block) x N, i.e. stored block column by block column (one
 * row of N values per block column), so that both the writer and the reader
 * touch whole memory lines.
 */
int32_t jf_add_q(const int8_t* X1, const float* S1, const int8_t* X2, const float* S2, int64_t N, int64_t C,
                 int32_t block, int8_t* Y, float* SY, float* row_mean, float* row_sumsq, void* stream);

/*
 * INT8 Dropout (App. A): Y = Q(X o m / (1 - p)) on the dequantized input.  The
 * keep mask m is an input (the random draw is the caller's): mask_bits is
 * N x (C/8) bytes, row-major, bit (c mod 8) of byte c/8 of a row belongs to
 * column c; 2-byte aligned.  0 <= p < 1 (else JF_ERR_SHAPE).  The backward
 * pass, dX = dY o m / (1 - p), is the same call on the upstream gradient.
 */
int32_t jf_dropout_q(const int8_t* X, const float* SX, const uint8_t* mask_bits, float p, int64_t N, int64_t C,
                     int32_t block, int8_t* Y, float* SY, void* stream);

/*
 * INT8 LayerNorm backward (standard LayerNorm gradient on dequantized
 * operands).  xhat = (x - mean) rstd, ghat = dY * gamma:
 *   dX = rstd (ghat - mean_C(ghat) - xhat mean_C(ghat xhat)),
 *   dgamma = sum_N dY xhat,  dbeta = sum_N dY   (FP32 [C], fixed summation order).
 * Needs jf_workspace_bytes(JF_OP_LAYERNORM_BWD, N, C, 0, block) bytes of ws
 * (at most 512 partial rows of dgamma | dbeta, and the two row means of every
 * row, which the pass hands from its first kernel to its second).
 */
int32_t jf_layernorm_q_bwd(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX, const float* gamma,
                           const float* mean, const float* rstd, int64_t N, int64_t C, int32_t block, int8_t* dX,
                           float* SdX, float* dgamma, float* dbeta, void* ws, size_t ws_bytes, void* stream);

/*
 * jf_layernorm_q_bwd for callers that cannot allocate device memory and so have
 * no workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and kernels as
 * jf_layernorm_q_bwd, bit for bit, without `ws` / `ws_bytes`: the partial rows
 * of dgamma | dbeta live in a static device array of JF_STATIC_SCRATCH_BYTES
 * inside the library (one copy per GPU, held until the process ends).  The call
 * allocates and frees nothing.  Problems whose
 * jf_workspace_bytes(JF_OP_LAYERNORM_BWD, N, C, 0, block) exceeds
 * JF_STATIC_SCRATCH_BYTES are rejected with JF_ERR_WORKSPACE (at C = 768 that
 * admits 655360 rows: 6 KiB per partial row, at most 512 of them, plus 8 bytes
 * per row).
 * All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams or threads) race; calls on one stream do not.
 * The first call on a device looks the array's address up
 * (hipGetSymbolAddress), so make it outside graph capture.
 */
#define JF_STATIC_SCRATCH_BYTES (8u << 20)
int32_t jf_layernorm_q_bwd_static(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX,
                                  const float* gamma, const float* mean, const float* rstd, int64_t N, int64_t C,
                                  int32_t block, int8_t* dX, float* SdX, float* dgamma, float* dbeta, void* stream);

/*
 * Test hook (Sec. 5.3, first equation): the INT32 product of K-block `kb`
 * for the whole output of one of the three GEMMs, computed by the same
 * staging / MFMA code as the production kernels.
 *   which 0: forward  (A = X N x C,  Bm = W D x C)   out N x D
 *   which 1: dgrad    (A = dY N x D, Bm = W D x C)   out N x C
 *   which 2: wgrad    (A = dY N x D, Bm = X N x C)   out D x C
 * out is INT32, dense row-major.
 */
int32_t jf_debug_linear_partials(int32_t which, const int8_t* A, const int8_t* Bm, int64_t N, int64_t C, int64_t D,
                                 int32_t block, int64_t kb, int32_t* out, void* stream);

/*
 * Test hook: force the tile shape of the GEMM entry points.  This is the one piece of state the library keeps
 * besides the last-error slot: a process-wide atomic integer, 0 (automatic) unless a test sets it, read once per
 * launch.  Production callers never call this.
 *   0 automatic (cost model), 1 128x128, 4 64x64, 6 256x128, 7 64x64 with a stage of 128 instead of 64 K bytes,
 *   8 128x64; other values: JF_ERR_SHAPE.
 * Shapes 7 and 8 exist for block 32 only; other blocks fall back to 128x128.  Block 128 knows 128x128 and
 * 256x128 only (automatic: 256x128 once the output has at least 256 such tiles).
 */
int32_t jf_debug_set_gemm_shape(int32_t shape);

#ifdef __cplusplus
}
#endif
#endif /* JETFIRE_H_ */
