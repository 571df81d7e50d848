// INT8-in / INT8-out GELU and LayerNorm, forward and backward (Sec. 6, Alg. 2, App. A).
//
// HBM-bound element-wise kernels.  Work is organised in strips of 8 rows x 128
// columns per wave instruction: lane = (row l/8, 16-byte column chunk l%8), so
// every row segment a wave touches is one full 128-byte line, loaded and stored
// as 16 bytes per lane.
#include "jf_common.hpp"

namespace jf {

__device__ __forceinline__ float std_normal_cdf(float x) { return 0.5f * erfcf(-0.70710678118654752f * x); }
__device__ __forceinline__ float std_normal_pdf(float x) { return 0.39894228040143268f * expf(-0.5f * x * x); }

struct GeluFwd {
  static constexpr bool kHasGrad = false;
  static __device__ __forceinline__ float apply(float x, float) { return x * std_normal_cdf(x); }
};
struct GeluBwd {
  static constexpr bool kHasGrad = true;
  static __device__ __forceinline__ float apply(float x, float g) { return g * (x * std_normal_pdf(x) + std_normal_cdf(x)); }
};

__device__ __forceinline__ void unpack16(const uint4& p, float s, float (&v)[16]) {
  const uint32_t w[4] = {p.x, p.y, p.z, p.w};
#pragma unroll
  for (int d = 0; d < 4; ++d)
#pragma unroll
    for (int b = 0; b < 4; ++b) v[4 * d + b] = byte_to_float(w[d], b) * s;
}

__device__ __forceinline__ uint4 quantize16(const float (&y)[16], float inv) {
  uint4 o;
  o.x = quantize4(y[0], y[1], y[2], y[3], inv);
  o.y = quantize4(y[4], y[5], y[6], y[7], inv);
  o.z = quantize4(y[8], y[9], y[10], y[11], inv);
  o.w = quantize4(y[12], y[13], y[14], y[15], inv);
  return o;
}

__device__ __forceinline__ float amax16(const float (&y)[16]) {
  float m = 0.0f;
#pragma unroll
  for (int e = 0; e < 16; ++e) m = fmaxf(m, fabsf(y[e]));
  return m;
}

// Reduce a per-lane value over the lanes of a wave that share a quantization block column:
// all 8 row lanes (bits 3..5) and the B/16 (<= 8) chunk lanes of the block (low bits).
template <int B>
__device__ __forceinline__ float strip_block_max(float m) {
  constexpr int CH = B >= 128 ? 7 : (B == 64 ? 3 : 1);
  return wave_group_max<56 | CH>(m);
}

// Element-wise operator of Alg. 2.  One workgroup (B/32 waves... fixed 4 waves) covers B rows x 128 columns:
// wave w handles rows [w*B/4, (w+1)*B/4) in B/32 passes of 8 rows.
template <typename Op, int B>
__global__ void __launch_bounds__(256) eltwise_kernel(const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                       const int8_t* __restrict__ G, const float* __restrict__ SG,
                                                       int rows, int cols, int8_t* __restrict__ Y,
                                                       float* __restrict__ SY) {
  constexpr int P = B / 32;  // 8-row passes per wave
  __shared__ float s_amax[4][4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ch = lane & 7, rsub = lane >> 3;
  const int c0 = blockIdx.x * 128, col = c0 + 16 * ch;
  const int r0 = blockIdx.y * B + wave * (B / 4);
  const bool col_ok = col < cols;  // cols % 32 == 0 and chunks are 16 wide: a 32-column group is all in or all out
  const int lc = cols / B;
  const int bj = col / B, bi = blockIdx.y;

  float y[P][16];
  float m = 0.0f;
  if (col_ok) {
    const float sx = SX[(int64_t)bi * lc + bj];
    const float sg = Op::kHasGrad ? SG[(int64_t)bi * lc + bj] : 0.0f;
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int row = r0 + 8 * p + rsub;
      const uint4 px = *reinterpret_cast<const uint4*>(X + (int64_t)row * cols + col);
      float x[16], gr[16];
      unpack16(px, sx, x);
      if (Op::kHasGrad) {
        const uint4 pg = *reinterpret_cast<const uint4*>(G + (int64_t)row * cols + col);
        unpack16(pg, sg, gr);
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) y[p][e] = Op::apply(x[e], Op::kHasGrad ? gr[e] : 0.0f);
      m = fmaxf(m, amax16(y[p]));
    }
  } else {
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
      for (int e = 0; e < 16; ++e) y[p][e] = 0.0f;
  }
  m = strip_block_max<B>(m);
  // s_amax[wave][32-column group]; for B >= 64 the in-wave reduction already covered the whole block width
  if ((lane & 57) == 0) s_amax[wave][ch >> 1] = m;
  __syncthreads();
  m = fmaxf(fmaxf(s_amax[0][ch >> 1], s_amax[1][ch >> 1]), fmaxf(s_amax[2][ch >> 1], s_amax[3][ch >> 1]));
  float scale, inv;
  block_scale(m, scale, inv);
  if (!col_ok) return;
  if (wave == 0 && rsub == 0 && (col % B) == 0) SY[(int64_t)bi * lc + bj] = scale;
#pragma unroll
  for (int p = 0; p < P; ++p) {
    const int row = r0 + 8 * p + rsub;
    *reinterpret_cast<uint4*>(Y + (int64_t)row * cols + col) = quantize16(y[p], inv);
  }
}

// ------------------------------------------------------------------ LayerNorm forward
// One workgroup owns B rows and all C columns.  Pass 1: exact per-(row, 16-column chunk) integer sums of
// codes and squared codes (v_dot4), scaled by the block scale and accumulated per row in FP64 -- the same
// row-partials scheme as App. A, computed from the INT8 input itself.  Pass 2: per 128-column group,
// normalise, find the block max-abs across the four waves, quantize, store.
template <int B>
__global__ void __launch_bounds__(256) layernorm_fwd_kernel(const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                             const float* __restrict__ gamma,
                                                             const float* __restrict__ beta, float eps, int rows,
                                                             int cols, int8_t* __restrict__ Y, float* __restrict__ SY,
                                                             float* __restrict__ mean_out, float* __restrict__ rstd_out) {
  constexpr int P = B / 32;
  __shared__ float s_amax[2][4][4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ch = lane & 7, rsub = lane >> 3;
  const int r0 = blockIdx.x * B + wave * (B / 4);
  const int lc = cols / B, bi = blockIdx.x;
  const int ngroups = (cols + 127) / 128;

  float mu[P], rs[P];
#pragma unroll
  for (int p = 0; p < P; ++p) {
    const int row = r0 + 8 * p + rsub;
    double sum = 0.0, sq = 0.0;
    for (int gidx = 0; gidx < ngroups; ++gidx) {
      const int col = gidx * 128 + 16 * ch;
      if (col < cols) {
        const uint4 px = *reinterpret_cast<const uint4*>(X + (int64_t)row * cols + col);
        const float sx = SX[(int64_t)bi * lc + col / B];
        int s1 = 0, s2 = 0;
        s1 = __builtin_amdgcn_sdot4((int)px.x, 0x01010101, s1, false);
        s1 = __builtin_amdgcn_sdot4((int)px.y, 0x01010101, s1, false);
        s1 = __builtin_amdgcn_sdot4((int)px.z, 0x01010101, s1, false);
        s1 = __builtin_amdgcn_sdot4((int)px.w, 0x01010101, s1, false);
        s2 = __builtin_amdgcn_sdot4((int)px.x, (int)px.x, s2, false);
        s2 = __builtin_amdgcn_sdot4((int)px.y, (int)px.y, s2, false);
        s2 = __builtin_amdgcn_sdot4((int)px.z, (int)px.z, s2, false);
        s2 = __builtin_amdgcn_sdot4((int)px.w, (int)px.w, s2, false);
        const double sd = (double)sx;
        sum += sd * (double)s1;
        sq += sd * sd * (double)s2;
      }
    }
    sum = wave_group_sum_f64<7>(sum);
    sq = wave_group_sum_f64<7>(sq);
    const double mean = sum / (double)cols;
    double var = sq / (double)cols - mean * mean;
    var = var > 0.0 ? var : 0.0;
    const double rstd = 1.0 / sqrt(var + (double)eps);
    mu[p] = (float)mean;
    rs[p] = (float)rstd;
    if (ch == 0) {
      mean_out[row] = mu[p];
      rstd_out[row] = rs[p];
    }
  }

  for (int gidx = 0; gidx < ngroups; ++gidx) {
    const int col = gidx * 128 + 16 * ch;
    const bool col_ok = col < cols;
    float y[P][16];
    float m = 0.0f;
    if (col_ok) {
      const float sx = SX[(int64_t)bi * lc + col / B];
      float gm[16], bt[16];
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const float4 g4 = *reinterpret_cast<const float4*>(gamma + col + 4 * d);
        const float4 b4 = *reinterpret_cast<const float4*>(beta + col + 4 * d);
        gm[4 * d] = g4.x; gm[4 * d + 1] = g4.y; gm[4 * d + 2] = g4.z; gm[4 * d + 3] = g4.w;
        bt[4 * d] = b4.x; bt[4 * d + 1] = b4.y; bt[4 * d + 2] = b4.z; bt[4 * d + 3] = b4.w;
      }
#pragma unroll
      for (int p = 0; p < P; ++p) {
        const int row = r0 + 8 * p + rsub;
        const uint4 px = *reinterpret_cast<const uint4*>(X + (int64_t)row * cols + col);
        float x[16];
        unpack16(px, sx, x);
#pragma unroll
        for (int e = 0; e < 16; ++e) y[p][e] = __builtin_fmaf((x[e] - mu[p]) * rs[p], gm[e], bt[e]);
        m = fmaxf(m, amax16(y[p]));
      }
    }
    m = strip_block_max<B>(m);
    const int buf = gidx & 1;
    if ((lane & 57) == 0) s_amax[buf][wave][ch >> 1] = m;
    __syncthreads();
    m = fmaxf(fmaxf(s_amax[buf][0][ch >> 1], s_amax[buf][1][ch >> 1]), fmaxf(s_amax[buf][2][ch >> 1], s_amax[buf][3][ch >> 1]));
    float scale, inv;
    block_scale(m, scale, inv);
    if (col_ok) {
      if (wave == 0 && rsub == 0 && (col % B) == 0) SY[(int64_t)bi * lc + col / B] = scale;
#pragma unroll
      for (int p = 0; p < P; ++p) {
        const int row = r0 + 8 * p + rsub;
        *reinterpret_cast<uint4*>(Y + (int64_t)row * cols + col) = quantize16(y[p], inv);
      }
    }
  }
}

// ------------------------------------------------------------------ LayerNorm backward
// Same ownership.  Pass 1: per row m1 = mean_C(ghat), m2 = mean_C(ghat * xhat); per column the partial
// sums of g * xhat and g over this workgroup's B rows go to the workspace (one row of partials per
// workgroup, summed in a fixed order by colsum_kernel).  Pass 2: dx, block max-abs, quantize, store.
template <int B>
__global__ void __launch_bounds__(256) layernorm_bwd_kernel(const int8_t* __restrict__ G, const float* __restrict__ SG,
                                                             const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                             const float* __restrict__ gamma,
                                                             const float* __restrict__ mean_in,
                                                             const float* __restrict__ rstd_in, int rows, int cols,
                                                             int8_t* __restrict__ dX, float* __restrict__ SdX,
                                                             float* __restrict__ partials) {
  constexpr int P = B / 32;
  __shared__ float s_amax[2][4][4];
  __shared__ float s_col[2][4][2][128];  // [buffer][wave][dgamma|dbeta][column of the group]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ch = lane & 7, rsub = lane >> 3;
  const int r0 = blockIdx.x * B + wave * (B / 4);
  const int lc = cols / B, bi = blockIdx.x;
  const int ngroups = (cols + 127) / 128;
  float* part_g = partials + (int64_t)blockIdx.x * 2 * cols;
  float* part_b = part_g + cols;

  float mu[P], rs[P], m1[P], m2[P];
#pragma unroll
  for (int p = 0; p < P; ++p) {
    const int row = r0 + 8 * p + rsub;
    mu[p] = mean_in[row];
    rs[p] = rstd_in[row];
    m1[p] = 0.0f;
    m2[p] = 0.0f;
  }
  for (int gidx = 0; gidx < ngroups; ++gidx) {
    const int col = gidx * 128 + 16 * ch;
    const bool col_ok = col < cols;
    float cg[16], cb[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) cg[e] = cb[e] = 0.0f;
    if (col_ok) {
      const float sx = SX[(int64_t)bi * lc + col / B], sg = SG[(int64_t)bi * lc + col / B];
      float gm[16];
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const float4 g4 = *reinterpret_cast<const float4*>(gamma + col + 4 * d);
        gm[4 * d] = g4.x; gm[4 * d + 1] = g4.y; gm[4 * d + 2] = g4.z; gm[4 * d + 3] = g4.w;
      }
#pragma unroll
      for (int p = 0; p < P; ++p) {
        const int row = r0 + 8 * p + rsub;
        const uint4 px = *reinterpret_cast<const uint4*>(X + (int64_t)row * cols + col);
        const uint4 pg = *reinterpret_cast<const uint4*>(G + (int64_t)row * cols + col);
        float x[16], gr[16];
        unpack16(px, sx, x);
        unpack16(pg, sg, gr);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float xh = (x[e] - mu[p]) * rs[p];
          const float gh = gr[e] * gm[e];
          m1[p] += gh;
          m2[p] = __builtin_fmaf(gh, xh, m2[p]);
          cg[e] = __builtin_fmaf(gr[e], xh, cg[e]);
          cb[e] += gr[e];
        }
      }
    }
    // column partials: sum over the 8 row lanes, then over the four waves in a fixed order
    const int buf = gidx & 1;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      cg[e] = wave_group_sum<56>(cg[e]);
      cb[e] = wave_group_sum<56>(cb[e]);
    }
    if (rsub == 0) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        s_col[buf][wave][0][16 * ch + e] = cg[e];
        s_col[buf][wave][1][16 * ch + e] = cb[e];
      }
    }
    __syncthreads();
    {
      const int which = threadIdx.x >> 7, c = threadIdx.x & 127;
      if (gidx * 128 + c < cols) {
        const float v = ((s_col[buf][0][which][c] + s_col[buf][1][which][c]) + s_col[buf][2][which][c]) + s_col[buf][3][which][c];
        (which ? part_b : part_g)[gidx * 128 + c] = v;
      }
    }
  }
#pragma unroll
  for (int p = 0; p < P; ++p) {
    m1[p] = wave_group_sum<7>(m1[p]) / (float)cols;
    m2[p] = wave_group_sum<7>(m2[p]) / (float)cols;
  }

  for (int gidx = 0; gidx < ngroups; ++gidx) {
    const int col = gidx * 128 + 16 * ch;
    const bool col_ok = col < cols;
    float y[P][16];
    float m = 0.0f;
    if (col_ok) {
      const float sx = SX[(int64_t)bi * lc + col / B], sg = SG[(int64_t)bi * lc + col / B];
      float gm[16];
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const float4 g4 = *reinterpret_cast<const float4*>(gamma + col + 4 * d);
        gm[4 * d] = g4.x; gm[4 * d + 1] = g4.y; gm[4 * d + 2] = g4.z; gm[4 * d + 3] = g4.w;
      }
#pragma unroll
      for (int p = 0; p < P; ++p) {
        const int row = r0 + 8 * p + rsub;
        const uint4 px = *reinterpret_cast<const uint4*>(X + (int64_t)row * cols + col);
        const uint4 pg = *reinterpret_cast<const uint4*>(G + (int64_t)row * cols + col);
        float x[16], gr[16];
        unpack16(px, sx, x);
        unpack16(pg, sg, gr);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float xh = (x[e] - mu[p]) * rs[p];
          const float gh = gr[e] * gm[e];
          y[p][e] = rs[p] * ((gh - m1[p]) - xh * m2[p]);
        }
        m = fmaxf(m, amax16(y[p]));
      }
    }
    m = strip_block_max<B>(m);
    const int buf = gidx & 1;
    if ((lane & 57) == 0) s_amax[buf][wave][ch >> 1] = m;
    __syncthreads();
    m = fmaxf(fmaxf(s_amax[buf][0][ch >> 1], s_amax[buf][1][ch >> 1]), fmaxf(s_amax[buf][2][ch >> 1], s_amax[buf][3][ch >> 1]));
    float scale, inv;
    block_scale(m, scale, inv);
    if (col_ok) {
      if (wave == 0 && rsub == 0 && (col % B) == 0) SdX[(int64_t)bi * lc + col / B] = scale;
#pragma unroll
      for (int p = 0; p < P; ++p) {
        const int row = r0 + 8 * p + rsub;
        *reinterpret_cast<uint4*>(dX + (int64_t)row * cols + col) = quantize16(y[p], inv);
      }
    }
  }
}

// dgamma / dbeta: sum the per-workgroup partial rows in ascending order (bit-stable from run to run).
__global__ void __launch_bounds__(256) colsum_kernel(const float* __restrict__ partials, int nparts, int cols,
                                                      float* __restrict__ dgamma, float* __restrict__ dbeta) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= 2 * cols) return;
  float acc = 0.0f;
  for (int p = 0; p < nparts; ++p) acc += partials[(int64_t)p * 2 * cols + c];
  if (c < cols) dgamma[c] = acc;
  else dbeta[c - cols] = acc;
}

template <typename Op>
static void launch_eltwise(int block, const int8_t* X, const float* SX, const int8_t* G, const float* SG, int rows,
                           int cols, int8_t* Y, float* SY, hipStream_t st) {
  dim3 grid((cols + 127) / 128, rows / block);
  if (block == 32) hipLaunchKernelGGL((eltwise_kernel<Op, 32>), grid, dim3(256), 0, st, X, SX, G, SG, rows, cols, Y, SY);
  else if (block == 64) hipLaunchKernelGGL((eltwise_kernel<Op, 64>), grid, dim3(256), 0, st, X, SX, G, SG, rows, cols, Y, SY);
  else hipLaunchKernelGGL((eltwise_kernel<Op, 128>), grid, dim3(256), 0, st, X, SX, G, SG, rows, cols, Y, SY);
}

static int32_t check_eltwise(const void* x, const void* sx, const void* y, const void* sy, int64_t N, int64_t C,
                             int32_t block) {
  if (!x || !sx || !y || !sy) return JF_ERR_NULL;
  if (!valid_block(block)) return JF_ERR_BLOCK;
  if (!valid_dim(N, block) || !valid_dim(C, block)) return JF_ERR_SHAPE;
  if (!aligned16(x) || !aligned4(sx) || !aligned16(y) || !aligned4(sy)) return JF_ERR_ALIGN;
  return JF_OK;
}

}  // namespace jf

extern "C" int32_t jf_gelu_q(const int8_t* X, const float* SX, int64_t N, int64_t C, int32_t block, int8_t* Y,
                             float* SY, void* stream) {
  using namespace jf;
  int32_t rc = check_eltwise(X, SX, Y, SY, N, C, block);
  if (rc != JF_OK) return rc;
  launch_eltwise<GeluFwd>(block, X, SX, nullptr, nullptr, (int)N, (int)C, Y, SY, reinterpret_cast<hipStream_t>(stream));
  return launch_status();
}

extern "C" int32_t jf_gelu_q_bwd(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX, int64_t N,
                                 int64_t C, int32_t block, int8_t* dX, float* SdX, void* stream) {
  using namespace jf;
  int32_t rc = check_eltwise(X, SX, dX, SdX, N, C, block);
  if (rc != JF_OK) return rc;
  if (!dY || !SdY) return JF_ERR_NULL;
  if (!aligned16(dY) || !aligned4(SdY)) return JF_ERR_ALIGN;
  launch_eltwise<GeluBwd>(block, X, SX, dY, SdY, (int)N, (int)C, dX, SdX, reinterpret_cast<hipStream_t>(stream));
  return launch_status();
}

extern "C" int32_t jf_layernorm_q(const int8_t* X, const float* SX, const float* gamma, const float* beta, float eps,
                                  int64_t N, int64_t C, int32_t block, int8_t* Y, float* SY, float* mean, float* rstd,
                                  void* stream) {
  using namespace jf;
  int32_t rc = check_eltwise(X, SX, Y, SY, N, C, block);
  if (rc != JF_OK) return rc;
  if (!gamma || !beta || !mean || !rstd) return JF_ERR_NULL;
  if (!aligned16(gamma) || !aligned16(beta) || !aligned4(mean) || !aligned4(rstd)) return JF_ERR_ALIGN;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  dim3 grid((unsigned)(N / block));
  if (block == 32) hipLaunchKernelGGL((layernorm_fwd_kernel<32>), grid, dim3(256), 0, st, X, SX, gamma, beta, eps, (int)N, (int)C, Y, SY, mean, rstd);
  else if (block == 64) hipLaunchKernelGGL((layernorm_fwd_kernel<64>), grid, dim3(256), 0, st, X, SX, gamma, beta, eps, (int)N, (int)C, Y, SY, mean, rstd);
  else hipLaunchKernelGGL((layernorm_fwd_kernel<128>), grid, dim3(256), 0, st, X, SX, gamma, beta, eps, (int)N, (int)C, Y, SY, mean, rstd);
  return launch_status();
}

extern "C" int32_t jf_layernorm_q_bwd(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX,
                                      const float* gamma, const float* mean, const float* rstd, int64_t N, int64_t C,
                                      int32_t block, int8_t* dX, float* SdX, float* dgamma, float* dbeta, void* ws,
                                      size_t ws_bytes, void* stream) {
  using namespace jf;
  int32_t rc = check_eltwise(X, SX, dX, SdX, N, C, block);
  if (rc != JF_OK) return rc;
  if (!dY || !SdY || !gamma || !mean || !rstd || !dgamma || !dbeta) return JF_ERR_NULL;
  if (!aligned16(dY) || !aligned4(SdY) || !aligned16(gamma) || !aligned4(mean) || !aligned4(rstd) ||
      !aligned4(dgamma) || !aligned4(dbeta))
    return JF_ERR_ALIGN;
  const size_t need = jf_workspace_bytes(JF_OP_LAYERNORM_BWD, N, C, 0, block);
  if (!ws || ws_bytes < need) return JF_ERR_WORKSPACE;
  if (!aligned16(ws)) return JF_ERR_ALIGN;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  float* partials = static_cast<float*>(ws);
  const int nparts = (int)(N / block);
  dim3 grid((unsigned)nparts);
  if (block == 32) hipLaunchKernelGGL((layernorm_bwd_kernel<32>), grid, dim3(256), 0, st, dY, SdY, X, SX, gamma, mean, rstd, (int)N, (int)C, dX, SdX, partials);
  else if (block == 64) hipLaunchKernelGGL((layernorm_bwd_kernel<64>), grid, dim3(256), 0, st, dY, SdY, X, SX, gamma, mean, rstd, (int)N, (int)C, dX, SdX, partials);
  else hipLaunchKernelGGL((layernorm_bwd_kernel<128>), grid, dim3(256), 0, st, dY, SdY, X, SX, gamma, mean, rstd, (int)N, (int)C, dX, SdX, partials);
  rc = launch_status();
  if (rc != JF_OK) return rc;
  hipLaunchKernelGGL(colsum_kernel, dim3((unsigned)((2 * C + 255) / 256)), dim3(256), 0, st, partials, nparts, (int)C, dgamma, dbeta);
  return launch_status();
}
