/*
 * CPU oracle for the per-block INT8 data flow of arxiv 2403.12422.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP kernels are checked against.  It shares no code, header, table or helper
 * with the GPU library, and the GPU library never calls into it.  Only the
 * test-suite, the smoke check and the CPU-baseline leg of the benchmark may
 * load the shared object built from this file.
 *
 * Everything follows the paper's notation:
 *   N tokens, C in-features, D out-features, B quantization block size,
 *   L_N = N/B etc. (Sec. 5.1).  A "per-block INT8 tensor" is a row-major INT8
 *   matrix of codes plus a dense row-major FP32 grid with one scale per BxB
 *   block (Sec. 4, Eq. 1; the paper stores FP16 scales, this build FP32).
 *
 * Readings of points the paper leaves open (each also listed in the design
 * notes of the repository):
 *   - scale  s = max|x| / 127 over the block, computed as one FP32 division
 *     (Sec. 4 ties the scale to the block maximum without giving a formula, Eq. 1
 *     divides by it; 127 makes the largest element map to +-127);
 *   - the round operator of Eq. 1 is round-half-to-even of the exact quotient,
 *     evaluated here in double (x and s are FP32 numbers);
 *   - an all-zero block gets s = 0 and all codes 0;
 *   - the FP32 accumulator of Sec. 5.3 / Alg. 1 is updated, per K-block k in
 *     ascending order, as  acc = fma(fl32(s_X * s_W), (float)Y_int32, acc);
 *     the same sum in double is returned beside it as the "exact" value;
 *   - the output quantizer of Alg. 1 (its last step before the store) is Eq. 1
 *     applied to that FP32 accumulator;
 *   - GELU uses the exact-erf form of App. A, LayerNorm uses biased variance,
 *     statistics of the dequantized INT8 input, and the standard gradient.
 *
 * Loops over independent output blocks / rows carry an OpenMP pragma; it does
 * not change any arithmetic or its order inside a block.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_SHAPE 2

int oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

static int bad_shape(int64_t rows, int64_t cols, int block) {
  return rows <= 0 || cols <= 0 || block <= 0 || rows % block || cols % block;
}

/* ------------------------------------------------------------------ */
/* Eq. 1, Sec. 4: the per-block quantizer Q.                           */
/* One block: amax, s = amax/127 (FP32), codes = round(x/s).           */
static void quantize_one_block(const float* x, int64_t ldx, int block, int8_t* q, int64_t ldq, float* s_out) {
  float amax = 0.0f;
  for (int i = 0; i < block; ++i)
    for (int j = 0; j < block; ++j) {
      float a = fabsf(x[i * ldx + j]);
      if (a > amax) amax = a;
    }
  if (amax == 0.0f) {
    *s_out = 0.0f;
    for (int i = 0; i < block; ++i)
      for (int j = 0; j < block; ++j) q[i * ldq + j] = 0;
    return;
  }
  volatile float s = amax / 127.0f; /* one IEEE FP32 division */
  *s_out = s;
  for (int i = 0; i < block; ++i)
    for (int j = 0; j < block; ++j) {
      double r = rint((double)x[i * ldx + j] / (double)s); /* FE_TONEAREST: ties to even */
      if (r > 127.0) r = 127.0;
      if (r < -127.0) r = -127.0;
      q[i * ldq + j] = (int8_t)r;
    }
}

/* Q on a whole rows x cols FP32 matrix (dense, row-major). */
int oracle_quantize_block(const float* x, int64_t rows, int64_t cols, int block, int8_t* q, float* s) {
  if (bad_shape(rows, cols, block)) return ORACLE_ERR_SHAPE;
  int64_t lr = rows / block, lc = cols / block;
#pragma omp parallel for collapse(2) schedule(static)
  for (int64_t bi = 0; bi < lr; ++bi)
    for (int64_t bj = 0; bj < lc; ++bj)
      quantize_one_block(x + bi * block * cols + bj * block, cols, block, q + bi * block * cols + bj * block, cols,
                         s + bi * lc + bj);
  return ORACLE_OK;
}

/* Eq. 1, Sec. 4: the dequantizer Q^-1, code * scale, returned exactly (double). */
int oracle_dequantize(const int8_t* q, const float* s, int64_t rows, int64_t cols, int block, double* out) {
  if (bad_shape(rows, cols, block)) return ORACLE_ERR_SHAPE;
  int64_t lc = cols / block;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t j = 0; j < cols; ++j) out[i * cols + j] = (double)q[i * cols + j] * (double)s[(i / block) * lc + j / block];
  return ORACLE_OK;
}

/* Transpose of a per-block tensor: codes and scale grid are both transposed.
 * Square blocks make this equal to quantizing the transposed source (Sec. 4:
 * the format must serve X W^T, dY W and dY^T X alike). */
int oracle_transpose(const int8_t* q, const float* s, int64_t rows, int64_t cols, int block, int8_t* qT, float* sT) {
  if (bad_shape(rows, cols, block)) return ORACLE_ERR_SHAPE;
  int64_t lr = rows / block, lc = cols / block;
  for (int64_t i = 0; i < rows; ++i)
    for (int64_t j = 0; j < cols; ++j) qT[j * rows + i] = q[i * cols + j];
  for (int64_t i = 0; i < lr; ++i)
    for (int64_t j = 0; j < lc; ++j) sT[j * lr + i] = s[i * lc + j];
  return ORACLE_OK;
}

/* ------------------------------------------------------------------ */
/* Sec. 5.3 first equation: the INT32 product of one pair of quantization
 * blocks, Y_int32 = A_{p,k} B_{q,k}^T, for K-block index kb and every output
 * block (p, q).  A is M x K, Bm is Nn x K (the "NT" form Y = X W^T of Eq. 2).
 * out is M x Nn INT32.                                                   */
int oracle_block_partials(const int8_t* A, const int8_t* Bm, int64_t M, int64_t Nn, int64_t K, int block, int64_t kb,
                          int32_t* out) {
  if (bad_shape(M, K, block) || bad_shape(Nn, K, block) || kb < 0 || kb >= K / block) return ORACLE_ERR_SHAPE;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < M; ++i)
    for (int64_t j = 0; j < Nn; ++j) {
      int32_t v = 0;
      for (int kk = 0; kk < block; ++kk) v += (int32_t)A[i * K + kb * block + kk] * (int32_t)Bm[j * K + kb * block + kk];
      out[i * Nn + j] = v;
    }
  return ORACLE_OK;
}

/* Alg. 1 (INT8 linear layer) in its canonical NT form out = A * Bm^T:
 *   for each output block (p,q), for k = 0 .. K/B-1 ascending:
 *     V   = A_{p,k} Bm_{q,k}^T            exact INT32           (Alg. 1, on-chip INT8 matmul)
 *     t   = fl32(S_A[p,k] * S_B[q,k])
 *     acc = fma(t, (float)V, acc)          FP32 accumulator      (Alg. 1, dequantize-and-accumulate)
 *   then Eq. 1 on the FP32 accumulator -> codes + S_out[p,q]     (Alg. 1, quantize the output)
 * acc32 (M x Nn, nullable) receives the FP32 accumulator, acc64 (nullable) the
 * same sum carried in double (products s_A*s_B exact, no FP32 rounding).     */
int oracle_linear_nt(const int8_t* A, const float* SA, const int8_t* Bm, const float* SB, int64_t M, int64_t Nn,
                     int64_t K, int block, int8_t* out_q, float* out_s, float* acc32, double* acc64) {
  if (bad_shape(M, K, block) || bad_shape(Nn, K, block)) return ORACLE_ERR_SHAPE;
  int64_t lm = M / block, ln = Nn / block, lk = K / block;
  int err = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int64_t p = 0; p < lm; ++p)
    for (int64_t q = 0; q < ln; ++q) {
      float* f32 = (float*)malloc(sizeof(float) * block * block);
      double* f64 = (double*)malloc(sizeof(double) * block * block);
      if (!f32 || !f64) {
#pragma omp atomic write
        err = 1;
        free(f32);
        free(f64);
        continue;
      }
      for (int e = 0; e < block * block; ++e) {
        f32[e] = 0.0f;
        f64[e] = 0.0;
      }
      for (int64_t k = 0; k < lk; ++k) {
        float sa = SA[p * lk + k], sb = SB[q * lk + k];
        volatile float t = sa * sb;
        double td = (double)sa * (double)sb;
        for (int i = 0; i < block; ++i) {
          const int8_t* arow = A + (p * block + i) * K + k * block;
          for (int j = 0; j < block; ++j) {
            const int8_t* brow = Bm + (q * block + j) * K + k * block;
            int32_t v = 0;
            for (int kk = 0; kk < block; ++kk) v += (int32_t)arow[kk] * (int32_t)brow[kk];
            f32[i * block + j] = fmaf(t, (float)v, f32[i * block + j]);
            f64[i * block + j] += td * (double)v;
          }
        }
      }
      if (out_q && out_s)
        quantize_one_block(f32, block, block, out_q + p * block * Nn + q * block, Nn, out_s + p * ln + q);
      for (int i = 0; i < block; ++i)
        for (int j = 0; j < block; ++j) {
          if (acc32) acc32[(p * block + i) * Nn + q * block + j] = f32[i * block + j];
          if (acc64) acc64[(p * block + i) * Nn + q * block + j] = f64[i * block + j];
        }
      free(f32);
      free(f64);
    }
  return err ? 3 : ORACLE_OK;
}

/* The same, but only for a list of output blocks (p[i], q[i]); used to check
 * full-size GPU results on a sample.  Outputs are packed per listed block:
 * out_q / acc32 / acc64 hold nblk consecutive BxB tiles, out_s nblk scales. */
int oracle_linear_nt_blocks(const int8_t* A, const float* SA, const int8_t* Bm, const float* SB, int64_t M, int64_t Nn,
                            int64_t K, int block, const int64_t* bp, const int64_t* bq, int64_t nblk, int8_t* out_q,
                            float* out_s, float* acc32, double* acc64) {
  if (bad_shape(M, K, block) || bad_shape(Nn, K, block)) return ORACLE_ERR_SHAPE;
  int64_t lk = K / block;
  int64_t bb = (int64_t)block * block;
  for (int64_t n = 0; n < nblk; ++n)
    if (bp[n] < 0 || bp[n] >= M / block || bq[n] < 0 || bq[n] >= Nn / block) return ORACLE_ERR_SHAPE;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t n = 0; n < nblk; ++n) {
    int64_t p = bp[n], q = bq[n];
    float* f32 = acc32 + n * bb;
    double* f64 = acc64 + n * bb;
    for (int64_t e = 0; e < bb; ++e) {
      f32[e] = 0.0f;
      f64[e] = 0.0;
    }
    for (int64_t k = 0; k < lk; ++k) {
      float sa = SA[p * lk + k], sb = SB[q * lk + k];
      volatile float t = sa * sb;
      double td = (double)sa * (double)sb;
      for (int i = 0; i < block; ++i) {
        const int8_t* arow = A + (p * block + i) * K + k * block;
        for (int j = 0; j < block; ++j) {
          const int8_t* brow = Bm + (q * block + j) * K + k * block;
          int32_t v = 0;
          for (int kk = 0; kk < block; ++kk) v += (int32_t)arow[kk] * (int32_t)brow[kk];
          f32[i * block + j] = fmaf(t, (float)v, f32[i * block + j]);
          f64[i * block + j] += td * (double)v;
        }
      }
    }
    quantize_one_block(f32, block, block, out_q + n * bb, block, out_s + n);
  }
  return ORACLE_OK;
}

/* Sec. 4, the three matrix products of a linear layer.  Each is Alg. 1 on
 * explicitly transposed per-block operands:
 *   forward   Y  = X W^T     : A = X (N x C),        Bm = W (D x C)
 *   dgrad     dX = dY W      : A = dY (N x D),       Bm = W^T (C x D)
 *   wgrad     dW = dY^T X    : A = dY^T (D x N),     Bm = X^T (C x N)       */
int oracle_linear_fwd(const int8_t* X, const float* SX, const int8_t* W, const float* SW, int64_t N, int64_t C,
                      int64_t D, int block, int8_t* Y, float* SY, float* Y32, double* Y64) {
  return oracle_linear_nt(X, SX, W, SW, N, D, C, block, Y, SY, Y32, Y64);
}

int oracle_linear_dgrad(const int8_t* dY, const float* SdY, const int8_t* W, const float* SW, int64_t N, int64_t C,
                        int64_t D, int block, int8_t* dX, float* SdX, float* dX32, double* dX64) {
  if (bad_shape(N, D, block) || bad_shape(D, C, block)) return ORACLE_ERR_SHAPE;
  int8_t* WT = (int8_t*)malloc((size_t)D * C);
  float* SWT = (float*)malloc(sizeof(float) * (D / block) * (C / block));
  if (!WT || !SWT) {
    free(WT);
    free(SWT);
    return 3;
  }
  oracle_transpose(W, SW, D, C, block, WT, SWT);
  int rc = oracle_linear_nt(dY, SdY, WT, SWT, N, C, D, block, dX, SdX, dX32, dX64);
  free(WT);
  free(SWT);
  return rc;
}

int oracle_linear_wgrad(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX, int64_t N, int64_t C,
                        int64_t D, int block, int8_t* dW, float* SdW, float* dW32, double* dW64) {
  if (bad_shape(N, D, block) || bad_shape(N, C, block)) return ORACLE_ERR_SHAPE;
  int8_t* dYT = (int8_t*)malloc((size_t)N * D);
  float* SdYT = (float*)malloc(sizeof(float) * (N / block) * (D / block));
  int8_t* XT = (int8_t*)malloc((size_t)N * C);
  float* SXT = (float*)malloc(sizeof(float) * (N / block) * (C / block));
  int rc = 3;
  if (dYT && SdYT && XT && SXT) {
    oracle_transpose(dY, SdY, N, D, block, dYT, SdYT);
    oracle_transpose(X, SX, N, C, block, XT, SXT);
    rc = oracle_linear_nt(dYT, SdYT, XT, SXT, D, C, N, block, dW, SdW, dW32, dW64);
  }
  free(dYT);
  free(SdYT);
  free(XT);
  free(SXT);
  return rc;
}

/* ------------------------------------------------------------------ */
/* Alg. 2 (INT8 non-linear operator) common tail: FP32 result -> Eq. 1. */
static int quantize_from_double(const double* y, int64_t rows, int64_t cols, int block, int8_t* q, float* s) {
  float* y32 = (float*)malloc(sizeof(float) * rows * cols);
  if (!y32) return 3;
  for (int64_t e = 0; e < rows * cols; ++e) y32[e] = (float)y[e]; /* the Y^FP32 of Alg. 2 */
  int rc = oracle_quantize_block(y32, rows, cols, block, q, s);
  free(y32);
  return rc;
}

static double std_normal_cdf(double x) { return 0.5 * (1.0 + erf(x / sqrt(2.0))); }
static double std_normal_pdf(double x) { return exp(-0.5 * x * x) / sqrt(2.0 * M_PI); }

/* App. A: GELU(x) = x * Phi(x) on the dequantized input, then Alg. 2's
 * quantize step.  y_f (nullable) receives the pre-quantization values. */
int oracle_gelu_q(const int8_t* X, const float* SX, int64_t N, int64_t C, int block, int8_t* Y, float* SY, double* y_f) {
  if (bad_shape(N, C, block)) return ORACLE_ERR_SHAPE;
  double* y = (double*)malloc(sizeof(double) * N * C);
  if (!y) return 3;
  oracle_dequantize(X, SX, N, C, block, y);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < N * C; ++e) y[e] = y[e] * std_normal_cdf(y[e]);
  if (y_f) memcpy(y_f, y, sizeof(double) * N * C);
  int rc = quantize_from_double(y, N, C, block, Y, SY);
  free(y);
  return rc;
}

/* App. A: dGELU/dx = x/sqrt(2 pi) * exp(-x^2/2) + Phi(x); dx = g * that,
 * with g and x both dequantized INT8 tensors. */
int oracle_gelu_q_bwd(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX, int64_t N, int64_t C,
                      int block, int8_t* dX, float* SdX, double* dx_f) {
  if (bad_shape(N, C, block)) return ORACLE_ERR_SHAPE;
  double* x = (double*)malloc(sizeof(double) * N * C);
  double* g = (double*)malloc(sizeof(double) * N * C);
  if (!x || !g) {
    free(x);
    free(g);
    return 3;
  }
  oracle_dequantize(X, SX, N, C, block, x);
  oracle_dequantize(dY, SdY, N, C, block, g);
#pragma omp parallel for schedule(static)
  for (int64_t e = 0; e < N * C; ++e) g[e] = g[e] * (x[e] * std_normal_pdf(x[e]) + std_normal_cdf(x[e]));
  if (dx_f) memcpy(dx_f, g, sizeof(double) * N * C);
  int rc = quantize_from_double(g, N, C, block, dX, SdX);
  free(x);
  free(g);
  return rc;
}

/* App. A, LayerNorm: row mean and (biased) variance of the dequantized input,
 * y = (x - mean) * rstd * gamma + beta, then Alg. 2's quantize step.
 * gamma and beta stay floating point (Sec. 7.1).  mean, rstd: FP32 per row. */
int oracle_layernorm_q(const int8_t* X, const float* SX, const float* gamma, const float* beta, float eps, int64_t N,
                       int64_t C, int block, int8_t* Y, float* SY, float* mean, float* rstd, double* y_f) {
  if (bad_shape(N, C, block)) return ORACLE_ERR_SHAPE;
  double* y = (double*)malloc(sizeof(double) * N * C);
  if (!y) return 3;
  oracle_dequantize(X, SX, N, C, block, y);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < N; ++i) {
    double* row = y + i * C;
    double mu = 0.0;
    for (int64_t j = 0; j < C; ++j) mu += row[j];
    mu /= (double)C;
    double var = 0.0;
    for (int64_t j = 0; j < C; ++j) var += (row[j] - mu) * (row[j] - mu);
    var /= (double)C;
    double rs = 1.0 / sqrt(var + (double)eps);
    for (int64_t j = 0; j < C; ++j) row[j] = (row[j] - mu) * rs * (double)gamma[j] + (double)beta[j];
    mean[i] = (float)mu;
    rstd[i] = (float)rs;
  }
  if (y_f) memcpy(y_f, y, sizeof(double) * N * C);
  int rc = quantize_from_double(y, N, C, block, Y, SY);
  free(y);
  return rc;
}

/* LayerNorm backward (the paper only says it follows the GELU pattern; this is
 * the standard gradient).  With xhat = (x - mean) * rstd and ghat = g * gamma:
 *   dx     = rstd * (ghat - mean_C(ghat) - xhat * mean_C(ghat * xhat))
 *   dgamma = sum_N g * xhat,   dbeta = sum_N g
 * x, g are dequantized INT8 tensors; mean, rstd are the saved FP32 vectors. */
int oracle_layernorm_q_bwd(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX, const float* gamma,
                           const float* mean, const float* rstd, int64_t N, int64_t C, int block, int8_t* dX,
                           float* SdX, float* dgamma, float* dbeta, double* dx_f) {
  if (bad_shape(N, C, block)) return ORACLE_ERR_SHAPE;
  double* x = (double*)malloc(sizeof(double) * N * C);
  double* g = (double*)malloc(sizeof(double) * N * C);
  double* dg = (double*)calloc(C, sizeof(double));
  double* db = (double*)calloc(C, sizeof(double));
  if (!x || !g || !dg || !db) {
    free(x);
    free(g);
    free(dg);
    free(db);
    return 3;
  }
  oracle_dequantize(X, SX, N, C, block, x);
  oracle_dequantize(dY, SdY, N, C, block, g);
  for (int64_t i = 0; i < N; ++i) { /* column sums in row order */
    double mu = (double)mean[i], rs = (double)rstd[i];
    for (int64_t j = 0; j < C; ++j) {
      double xh = (x[i * C + j] - mu) * rs;
      dg[j] += g[i * C + j] * xh;
      db[j] += g[i * C + j];
    }
  }
  for (int64_t j = 0; j < C; ++j) {
    dgamma[j] = (float)dg[j];
    dbeta[j] = (float)db[j];
  }
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < N; ++i) {
    double mu = (double)mean[i], rs = (double)rstd[i];
    double m1 = 0.0, m2 = 0.0;
    for (int64_t j = 0; j < C; ++j) {
      double xh = (x[i * C + j] - mu) * rs;
      double gh = g[i * C + j] * (double)gamma[j];
      m1 += gh;
      m2 += gh * xh;
    }
    m1 /= (double)C;
    m2 /= (double)C;
    for (int64_t j = 0; j < C; ++j) {
      double xh = (x[i * C + j] - mu) * rs;
      double gh = g[i * C + j] * (double)gamma[j];
      g[i * C + j] = rs * (gh - m1 - xh * m2);
    }
  }
  if (dx_f) memcpy(dx_f, g, sizeof(double) * N * C);
  int rc = quantize_from_double(g, N, C, block, dX, SdX);
  free(x);
  free(g);
  free(dg);
  free(db);
  return rc;
}

/* ------------------------------------------------------------------ */
/* App. A, Add: y = x1 + x2 on the dequantized operands (the residual
 * connection forward, and dx = df(y) + dy backward), then Alg. 2's quantize
 * step.  The modified ADD of App. A (LayerNorm paragraph) also stores, for
 * every row i and every block column j, the mean and the sum of squares of the
 * FP32 sum over the B columns of that block: row_mean, row_sumsq are N x C/B
 * FP32 matrices (both nullable).  y_f (nullable) receives the double sum. */
int oracle_add_q(const int8_t* X1, const float* S1, const int8_t* X2, const float* S2, int64_t N, int64_t C, int block,
                 int8_t* Y, float* SY, float* row_mean, float* row_sumsq, double* y_f) {
  if (bad_shape(N, C, block)) return ORACLE_ERR_SHAPE;
  double* a = (double*)malloc(sizeof(double) * N * C);
  double* b = (double*)malloc(sizeof(double) * N * C);
  if (!a || !b) {
    free(a);
    free(b);
    return 3;
  }
  oracle_dequantize(X1, S1, N, C, block, a);
  oracle_dequantize(X2, S2, N, C, block, b);
  for (int64_t e = 0; e < N * C; ++e) a[e] += b[e];
  const int64_t lc = C / block;
  if (row_mean || row_sumsq) {
    for (int64_t i = 0; i < N; ++i)
      for (int64_t j = 0; j < lc; ++j) {
        double s = 0.0, q = 0.0;
        for (int c = 0; c < block; ++c) {
          /* statistics of the FP32 values that Alg. 2 hands to the quantizer */
          double v = (double)(float)a[i * C + j * block + c];
          s += v;
          q += v * v;
        }
        if (row_mean) row_mean[i * lc + j] = (float)(s / (double)block);
        if (row_sumsq) row_sumsq[i * lc + j] = (float)q;
      }
  }
  if (y_f) memcpy(y_f, a, sizeof(double) * N * C);
  int rc = quantize_from_double(a, N, C, block, Y, SY);
  free(a);
  free(b);
  return rc;
}

/* App. A (LayerNorm paragraph): row statistics from ADD's partials.  With L_C = C/B block columns,
 *   mean_i = (1/L_C) sum_j row_mean[i][j],   E[x^2]_i = (1/C) sum_j row_sumsq[i][j],
 *   var_i = E[x^2]_i - mean_i^2 (biased, clamped at 0),   rstd_i = 1/sqrt(var_i + eps). */
int oracle_row_stats_from_partials(const float* row_mean, const float* row_sumsq, int64_t N, int64_t C, int block,
                                   float eps, float* mean, float* rstd) {
  if (bad_shape(N, C, block)) return ORACLE_ERR_SHAPE;
  const int64_t lc = C / block;
  for (int64_t i = 0; i < N; ++i) {
    double s = 0.0, q = 0.0;
    for (int64_t j = 0; j < lc; ++j) {
      s += (double)row_mean[i * lc + j];
      q += (double)row_sumsq[i * lc + j];
    }
    double mu = s / (double)lc;
    double var = q / (double)C - mu * mu;
    if (var < 0.0) var = 0.0;
    mean[i] = (float)mu;
    rstd[i] = (float)(1.0 / sqrt(var + (double)eps));
  }
  return ORACLE_OK;
}

/* App. A: LayerNorm that is handed its row statistics (FP32 mean, rstd) instead of computing them:
 * y = (x - mean) * rstd * gamma + beta on the dequantized input, then Alg. 2's quantize step. */
int oracle_layernorm_q_stats(const int8_t* X, const float* SX, const float* gamma, const float* beta, const float* mean,
                             const float* rstd, int64_t N, int64_t C, int block, int8_t* Y, float* SY, double* y_f) {
  if (bad_shape(N, C, block)) return ORACLE_ERR_SHAPE;
  double* y = (double*)malloc(sizeof(double) * N * C);
  if (!y) return 3;
  oracle_dequantize(X, SX, N, C, block, y);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < N; ++i)
    for (int64_t j = 0; j < C; ++j)
      y[i * C + j] = (y[i * C + j] - (double)mean[i]) * (double)rstd[i] * (double)gamma[j] + (double)beta[j];
  if (y_f) memcpy(y_f, y, sizeof(double) * N * C);
  int rc = quantize_from_double(y, N, C, block, Y, SY);
  free(y);
  return rc;
}

/* App. A, Dropout: Drop(x) = x o m / (1 - p) with a 0/1 mask m, and dDrop/dx = m / (1 - p): the backward pass
 * applies the same operator, with the same mask, to the upstream gradient.  The mask is an input (the random
 * draw is not part of the operator): bit (c mod 8) of byte mask[i * C/8 + c/8] belongs to element (i, c).
 * x is the dequantized INT8 input; the result goes through Alg. 2's quantize step. */
int oracle_dropout_q(const int8_t* X, const float* SX, const uint8_t* mask, float p, int64_t N, int64_t C, int block,
                     int8_t* Y, float* SY, double* y_f) {
  if (bad_shape(N, C, block)) return ORACLE_ERR_SHAPE;
  if (!(p >= 0.0f && p < 1.0f)) return ORACLE_ERR_SHAPE;
  double* y = (double*)malloc(sizeof(double) * N * C);
  if (!y) return 3;
  oracle_dequantize(X, SX, N, C, block, y);
  const double keep_scale = 1.0 / (1.0 - (double)p);
  for (int64_t i = 0; i < N; ++i)
    for (int64_t c = 0; c < C; ++c) {
      const int m = (mask[i * (C / 8) + c / 8] >> (c % 8)) & 1;
      y[i * C + c] = m ? y[i * C + c] * keep_scale : 0.0;
    }
  if (y_f) memcpy(y_f, y, sizeof(double) * N * C);
  int rc = quantize_from_double(y, N, C, block, Y, SY);
  free(y);
  return rc;
}
