// INT8-in / INT8-out LayerNorm, forward and backward (App. A).
//
// Block size 32: each pass is a small kernel that only leaves sums (row statistics forward; row means and
// dgamma | dbeta partial rows backward) followed by an element-wise operator on the 32 x 128 strips of jf_rowops.hpp, so no
// workgroup holds a row in registers and rows may be of any width.  Row sums of the forward pass come from exact integer
// dot products of the codes (v_dot4), scaled per block -- the row-partials scheme of App. A applied to the INT8 input
// itself -- or from the partials that the preceding Add wrote.  Block sizes 64 and 128 use one workgroup per B whole rows.
#include <algorithm>
#include <mutex>

#include "jf_rowops.hpp"

namespace jf {

// ------------------------------------------------------------------------------------------------
// Block sizes 64 and 128: one workgroup owns B rows and all C columns (C <= 4096), each wave a few of the rows.
// Lane l of a wave owns the 16-byte chunks l, l+64, ... of each of its rows, so a row is read as contiguous 1 KB
// runs and per-column quantities (gamma, beta, column sums) stay in registers while the wave walks down its
// rows.  NIT = ceil(C / 1024) chunks per lane and row.

// exact sums of the 16 codes of a chunk and of their squares
__device__ __forceinline__ void chunk_moments(const uint4& p, int& s1, int& s2) {
  s1 = __builtin_amdgcn_sdot4((int)p.x, 0x01010101, 0, false);
  s1 = __builtin_amdgcn_sdot4((int)p.y, 0x01010101, s1, false);
  s1 = __builtin_amdgcn_sdot4((int)p.z, 0x01010101, s1, false);
  s1 = __builtin_amdgcn_sdot4((int)p.w, 0x01010101, s1, false);
  s2 = __builtin_amdgcn_sdot4((int)p.x, (int)p.x, 0, false);
  s2 = __builtin_amdgcn_sdot4((int)p.y, (int)p.y, s2, false);
  s2 = __builtin_amdgcn_sdot4((int)p.z, (int)p.z, s2, false);
  s2 = __builtin_amdgcn_sdot4((int)p.w, (int)p.w, s2, false);
}

// Forward: NW = 16 waves per workgroup (a workgroup is alone on its compute unit, since there are only
// N/B of them), RW = B/16 rows per wave.  If the wave's rows fit in registers (KEEP) they are read once.
// FROM_PARTIALS: the row statistics come from the row partials of the preceding Add (row_mean, row_sumsq) instead
// of the codes.
template <int B, int NIT, bool FROM_PARTIALS>
__global__ void __launch_bounds__(1024) layernorm_fwd_kernel(const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                              const float* __restrict__ gamma,
                                                              const float* __restrict__ beta, float eps, int rows,
                                                              int cols, int8_t* __restrict__ Y, float* __restrict__ SY,
                                                              float* __restrict__ mean_out, float* __restrict__ rstd_out,
                                                              const float* __restrict__ row_mean,
                                                              const float* __restrict__ row_sumsq) {
  constexpr int NW = 16, RW = B / NW;
  constexpr bool KEEP = RW * NIT <= 8;
  const double inv_cols = 1.0 / (double)cols;  // uniform: one division per wave
  extern __shared__ float s_dyn[];  // [NW][C/32] per-wave block max-abs
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r0 = blockIdx.x * B + wave * RW;
  const int lc = cols / B, bi = blockIdx.x, nchunks = cols / 16, ngran = cols / 32;
  float* s_amax = s_dyn;

  bool ok[NIT];
  float sx[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int c = lane + 64 * it;
    ok[it] = c < nchunks;
    sx[it] = ok[it] ? SX[(int64_t)bi * lc + (16 * c) / B] : 0.0f;
  }
  uint4 xs[KEEP ? RW : 1][NIT];
  auto chunk = [&](int r, int it) -> uint4 {
    if (KEEP) return xs[r][it];
    return *reinterpret_cast<const uint4*>(X + (int64_t)(r0 + r) * cols + 16 * (lane + 64 * it));
  };
  if (KEEP) {
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
      for (int it = 0; it < NIT; ++it)
        xs[r][it] = ok[it] ? *reinterpret_cast<const uint4*>(X + (int64_t)(r0 + r) * cols + 16 * (lane + 64 * it))
                           : make_uint4(0, 0, 0, 0);
  }

  // sweep 1: row statistics.  Per 16-code chunk the sum and the sum of squares of the codes are exact integers
  // (v_dot4); times the block scale, in double, they are the chunk's contribution to the row sum and to the
  // row's sum of squares.  The row mean is reduced over the wave in FP32.  The variance is then taken about
  // that mean chunk by chunk, sum_c (x_c - mu)^2 = q - 2 mu s + n mu^2 in double -- the only place where large
  // terms cancel -- so that the per-lane partial sums are sums of non-negative terms, which FP32 reduces over
  // the wave without loss.  (Two FP32 butterflies instead of two FP64 ones: a quarter of the instructions.)
  float k1[RW][NIT], k2[RW];  // xhat = u * k1 + k2 with u = code + 128
  const float inv_cols_f = (float)inv_cols;
  // Statistics handed over by the preceding Add (App. A): per row and block column the mean and the sum of squares
  // over the block's B columns.  All of the wave's rows are requested at once, beside the codes.
  constexpr int NJ = (NIT * 1024 / B + 63) / 64;  // block columns per lane
  float pm[RW][NJ], pq[RW][NJ];
  if constexpr (FROM_PARTIALS) {
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
      for (int jj = 0; jj < NJ; ++jj) {
        const int j = lane + 64 * jj;
        pm[r][jj] = j < lc ? row_mean[(int64_t)(r0 + r) * lc + j] : 0.0f;
        pq[r][jj] = j < lc ? row_sumsq[(int64_t)(r0 + r) * lc + j] : 0.0f;
      }
  }
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    double cs[NIT], cq[NIT];  // per chunk: sum and sum of squares of the dequantized values
    double ds = 0.0;
    if constexpr (FROM_PARTIALS) {
#pragma unroll
      for (int jj = 0; jj < NJ; ++jj) ds += (double)B * (double)pm[r][jj];  // a block's sum is B times its mean
    } else {
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        cs[it] = cq[it] = 0.0;
        if (ok[it]) {
          int s1, s2;
          chunk_moments(chunk(r, it), s1, s2);
          const double sd = (double)sx[it];
          cs[it] = sd * (double)s1;
          cq[it] = sd * sd * (double)s2;
          ds += cs[it];
        }
      }
    }
    const float mu = wave_group_sum<63>((float)ds) * inv_cols_f;
    const double mud = (double)mu;
    double dv = 0.0;
    if constexpr (FROM_PARTIALS) {
#pragma unroll
      for (int jj = 0; jj < NJ; ++jj)
        if (lane + 64 * jj < lc)
          dv += (double)pq[r][jj] - 2.0 * mud * ((double)B * (double)pm[r][jj]) + (double)B * mud * mud;
    } else {
#pragma unroll
      for (int it = 0; it < NIT; ++it)
        if (ok[it]) dv += cq[it] - 2.0 * mud * cs[it] + 16.0 * mud * mud;
    }
    const float var = fmaxf(wave_group_sum<63>((float)dv) * inv_cols_f, 0.0f);
    // reciprocal square root: hardware approximation refined by one Newton step (relative error ~1e-7)
    const float ve = var + eps;
    float rs = __builtin_amdgcn_rsqf(ve);
    rs = rs * __builtin_fmaf(-0.5f * ve * rs, rs, 1.5f);
    if (lane == 0) {
      mean_out[r0 + r] = mu;
      rstd_out[r0 + r] = rs;
    }
#pragma unroll
    for (int it = 0; it < NIT; ++it) k1[r][it] = sx[it] * rs;
    k2[r] = -mu * rs;
  }

  // sweep 2: y = xhat * gamma + beta and its block max-abs.  With at most four chunks per lane the values
  // stay in registers (KEEPY); otherwise sweep 3 recomputes them.
  constexpr bool KEEPY = KEEP && RW * NIT <= 4;
  constexpr int LM = B / 16 - 1;  // lanes of one block column: mask 1, 3 or 7
  float ys[KEEPY ? RW : 1][KEEPY ? NIT : 1][16];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    float m = 0.0f;
    if (ok[it]) {
      float gm[16], bt[16];
      load16f(gamma + 16 * (lane + 64 * it), gm);
      load16f(beta + 16 * (lane + 64 * it), bt);
#pragma unroll
      for (int r = 0; r < RW; ++r) {
        float u[16];
        unpack16_biased(chunk(r, it), u);
        const float kb = __builtin_fmaf(-128.0f, k1[r][it], k2[r]);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float y = __builtin_fmaf(__builtin_fmaf(u[e], k1[r][it], kb), gm[e], bt[e]);
          if (KEEPY) ys[r][it][e] = y;
          m = fmaxf(m, fabsf(y));
        }
      }
    }
    m = wave_group_max<LM>(m);
    const int c = lane + 64 * it;
    if (ok[it] && (c & 1) == 0) s_amax[wave * ngran + (c >> 1)] = m;
  }
  __syncthreads();

  // sweep 3: quantize (recomputing y if it was not kept), store
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int c = lane + 64 * it;
    if (ok[it]) {
      float mm = 0.0f, scale;
      double inv;
#pragma unroll
      for (int w = 0; w < NW; ++w) mm = fmaxf(mm, s_amax[w * ngran + (c >> 1)]);
      block_scale(mm, scale, inv);
      if (wave == 0 && ((16 * c) % B) == 0) SY[(int64_t)bi * lc + (16 * c) / B] = scale;
      if (KEEPY) {
#pragma unroll
        for (int r = 0; r < RW; ++r)
          *reinterpret_cast<uint4*>(Y + (int64_t)(r0 + r) * cols + 16 * c) = quantize16(ys[r][it], inv);
      } else {
        float gm[16], bt[16];
        load16f(gamma + 16 * c, gm);
        load16f(beta + 16 * c, bt);
#pragma unroll
        for (int r = 0; r < RW; ++r) {
          float u[16], y[16];
          unpack16_biased(chunk(r, it), u);
          const float kb = __builtin_fmaf(-128.0f, k1[r][it], k2[r]);
#pragma unroll
          for (int e = 0; e < 16; ++e) y[e] = __builtin_fmaf(__builtin_fmaf(u[e], k1[r][it], kb), gm[e], bt[e]);
          *reinterpret_cast<uint4*>(Y + (int64_t)(r0 + r) * cols + 16 * c) = quantize16(y, inv);
        }
      }
    }
  }
}

// LayerNorm backward.  Eight waves per workgroup, RW = B/8 rows per wave, walked one row at a time (the next
// row's codes are requested before the current row is worked on).  A workgroup walks over the row blocks
// blockIdx.x, blockIdx.x + gridDim.x, ... and leaves ONE row of dgamma | dbeta partial sums in the
// workspace.  With ghat = g gamma and xhat = (x - mean) rstd, dx = rstd y where
//   y = ghat - mean_C(ghat) - xhat mean_C(ghat xhat).
// Pass A, per row: the two row means (wave reduction), the running column sums of g*xhat and g, and the
// max-abs of dx per chunk column; the row means go to LDS.  After the block max-abs is known, pass B reads
// the codes again (they are in L2), recomputes y and stores the codes.  The column sums stay in registers
// over all row blocks of the workgroup and are folded over the waves once, at the end, in a fixed order
// (wave w into LDS row w % 4 in round w / 4), so results are bit-stable.  NIT <= 2 (C <= 2048).
template <int B, int NIT>
__global__ void __launch_bounds__(512, NIT == 1 ? 3 : 2) layernorm_bwd_kernel(
    const int8_t* __restrict__ G, const float* __restrict__ SG, const int8_t* __restrict__ X, const float* __restrict__ SX,
    const float* __restrict__ gamma, const float* __restrict__ mean_in, const float* __restrict__ rstd_in, int rows,
    int cols, int8_t* __restrict__ dX, float* __restrict__ SdX, float* __restrict__ partials) {
  constexpr int NW = 8, RW = B / NW;
  extern __shared__ float s_dyn[];        // [NW][C/32] block max-abs | [B][2] row means | [4][2][C] column sums
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lc = cols / B, nchunks = cols / 16, ngran = cols / 32;
  float* s_amax = s_dyn;
  float* s_q = s_dyn + NW * ngran;
  float* s_col = s_q + 2 * B;
  const float inv_cols = 1.0f / (float)cols;

  bool ok[NIT];
  float gm[NIT][16], cgs[NIT][16], cbs[NIT][16];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    ok[it] = lane + 64 * it < nchunks;
#pragma unroll
    for (int e = 0; e < 16; ++e) gm[it][e] = cgs[it][e] = cbs[it][e] = 0.0f;
    if (ok[it]) load16f(gamma + 16 * (lane + 64 * it), gm[it]);
  }
  auto load_row = [&](const int8_t* base, int row, uint4 (&v)[NIT]) {
#pragma unroll
    for (int it = 0; it < NIT; ++it)
      v[it] = ok[it] ? *reinterpret_cast<const uint4*>(base + (int64_t)row * cols + 16 * (lane + 64 * it)) : make_uint4(0, 0, 0, 0);
  };

  // row statistics are the same for all lanes of a wave: scalar loads (the vectors are not written by this kernel)
  typedef const __attribute__((address_space(4))) float* const_f32_ptr;
  const const_f32_ptr mean_c = (const_f32_ptr)mean_in, rstd_c = (const_f32_ptr)rstd_in;
  for (int bi = blockIdx.x; bi < rows / B; bi += gridDim.x) {
    const int r0 = bi * B + wave * RW;
    const int r0u = __builtin_amdgcn_readfirstlane(r0);
    float sx[NIT], sgv[NIT], mloc[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + 64 * it;
      sx[it] = ok[it] ? SX[(int64_t)bi * lc + (16 * c) / B] : 0.0f;
      sgv[it] = ok[it] ? SG[(int64_t)bi * lc + (16 * c) / B] : 0.0f;
      mloc[it] = 0.0f;
    }

    // ---- pass A
    uint4 nx[NIT], ng[NIT];
    load_row(X, r0, nx);
    load_row(G, r0, ng);
#pragma unroll 1
    for (int r = 0; r < RW; ++r) {
      uint4 cx[NIT], cgc[NIT];
#pragma unroll
      for (int it = 0; it < NIT; ++it) { cx[it] = nx[it]; cgc[it] = ng[it]; }
      if (r + 1 < RW) {
        load_row(X, r0 + r + 1, nx);
        load_row(G, r0 + r + 1, ng);
      }
      const float mu = mean_c[r0u + r], rs = rstd_c[r0u + r];
      const float mrs = -mu * rs;
      float m1 = 0.0f, m2 = 0.0f;
      float xh[NIT][16], gh[NIT][16];
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        float ux[16], ug[16];
        unpack16_biased(cx[it], ux);
        unpack16_biased(cgc[it], ug);
        const float kx = sx[it] * rs, cx0 = __builtin_fmaf(-128.0f, kx, mrs);
        const float g128 = -128.0f * sgv[it];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          xh[it][e] = __builtin_fmaf(ux[e], kx, cx0);
          const float gv = __builtin_fmaf(ug[e], sgv[it], g128);
          gh[it][e] = gv * gm[it][e];
          m1 += gh[it][e];
          m2 = __builtin_fmaf(gh[it][e], xh[it][e], m2);
          cgs[it][e] = __builtin_fmaf(gv, xh[it][e], cgs[it][e]);
          cbs[it][e] += gv;
        }
      }
      const float q1 = wave_group_sum<63>(m1) * inv_cols;
      const float q2 = wave_group_sum<63>(m2) * inv_cols;
      if (lane == 0) {
        s_q[2 * (wave * RW + r)] = q1;
        s_q[2 * (wave * RW + r) + 1] = q2;
      }
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        float m = 0.0f;
#pragma unroll
        for (int e = 0; e < 16; ++e) m = fmaxf(m, fabsf(__builtin_fmaf(-xh[it][e], q2, gh[it][e] - q1)));
        mloc[it] = fmaxf(mloc[it], m * rs);
      }
    }
    constexpr int LM = B / 16 - 1;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const float m = wave_group_max<LM>(mloc[it]);
      const int c = lane + 64 * it;
      if (ok[it] && (c & 1) == 0) s_amax[wave * ngran + (c >> 1)] = m;
    }
    __syncthreads();

    // ---- pass B
    double inv[NIT];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int c = lane + 64 * it;
      float mm = 0.0f, scale;
      if (ok[it]) {
#pragma unroll
        for (int w = 0; w < NW; ++w) mm = fmaxf(mm, s_amax[w * ngran + (c >> 1)]);
      }
      block_scale(mm, scale, inv[it]);
      if (ok[it] && wave == 0 && ((16 * c) % B) == 0) SdX[(int64_t)bi * lc + (16 * c) / B] = scale;
    }
    load_row(X, r0, nx);
    load_row(G, r0, ng);
#pragma unroll 1
    for (int r = 0; r < RW; ++r) {
      uint4 cx[NIT], cgc[NIT];
#pragma unroll
      for (int it = 0; it < NIT; ++it) { cx[it] = nx[it]; cgc[it] = ng[it]; }
      if (r + 1 < RW) {
        load_row(X, r0 + r + 1, nx);
        load_row(G, r0 + r + 1, ng);
      }
      const float mu = mean_c[r0u + r], rs = rstd_c[r0u + r];
      const float mrs = -mu * rs;
      const float q1 = s_q[2 * (wave * RW + r)], q2 = s_q[2 * (wave * RW + r) + 1];
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        if (!ok[it]) continue;
        float ux[16], ug[16], y[16];
        unpack16_biased(cx[it], ux);
        unpack16_biased(cgc[it], ug);
        const float kx = sx[it] * rs, cx0 = __builtin_fmaf(-128.0f, kx, mrs);
        const float g128 = -128.0f * sgv[it];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float xhv = __builtin_fmaf(ux[e], kx, cx0);
          const float ghv = __builtin_fmaf(ug[e], sgv[it], g128) * gm[it][e];
          y[e] = __builtin_fmaf(-xhv, q2, ghv - q1) * rs;
        }
        *reinterpret_cast<uint4*>(dX + (int64_t)(r0 + r) * cols + 16 * (lane + 64 * it)) = quantize16(y, inv[it]);
      }
    }
    __syncthreads();  // max-abs slots and row means are rewritten by the next row block
  }

  // fold the column sums over the waves: wave w adds into LDS row w % 4 in round w / 4
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
#pragma unroll
    for (int round = 0; round < NW / 4; ++round) {
      if ((wave >> 2) == round && ok[it]) {
        float* row_g = s_col + (wave & 3) * 2 * cols + 16 * (lane + 64 * it);
        float* row_b = row_g + cols;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          float4 a = make_float4(cgs[it][4 * d], cgs[it][4 * d + 1], cgs[it][4 * d + 2], cgs[it][4 * d + 3]);
          float4 b = make_float4(cbs[it][4 * d], cbs[it][4 * d + 1], cbs[it][4 * d + 2], cbs[it][4 * d + 3]);
          if (round > 0) {
            const float4 pa = *reinterpret_cast<const float4*>(row_g + 4 * d);
            const float4 pb = *reinterpret_cast<const float4*>(row_b + 4 * d);
            a = make_float4(pa.x + a.x, pa.y + a.y, pa.z + a.z, pa.w + a.w);
            b = make_float4(pb.x + b.x, pb.y + b.y, pb.z + b.z, pb.w + b.w);
          }
          *reinterpret_cast<float4*>(row_g + 4 * d) = a;
          *reinterpret_cast<float4*>(row_b + 4 * d) = b;
        }
      }
      __syncthreads();
    }
  }
  {  // the four folded rows, added in a fixed order -> one row of the workspace
    float* dst = partials + (int64_t)blockIdx.x * 2 * cols;
    for (int i = threadIdx.x; i < 2 * cols / 4; i += 64 * NW) {
      const float4 a = *reinterpret_cast<const float4*>(s_col + 4 * i);
      const float4 b = *reinterpret_cast<const float4*>(s_col + 2 * cols + 4 * i);
      const float4 c = *reinterpret_cast<const float4*>(s_col + 4 * cols + 4 * i);
      const float4 d = *reinterpret_cast<const float4*>(s_col + 6 * cols + 4 * i);
      *reinterpret_cast<float4*>(dst + 4 * i) =
          make_float4((a.x + b.x) + (c.x + d.x), (a.y + b.y) + (c.y + d.y), (a.z + b.z) + (c.z + d.z), (a.w + b.w) + (c.w + d.w));
    }
  }
}

// LayerNorm backward for rows wider than 2048 columns (a lane owns up to four chunk columns, too many for
// running column sums in registers).  Sixteen waves per workgroup, RW = B/16 rows per wave.  Sweep 1: per row
// m1 = mean_C(ghat), m2 = mean_C(ghat xhat), and per column the sums of g*xhat and g over the wave's rows;
// the sixteen waves fold those column sums into four LDS rows in a fixed order (wave w adds into row w % 4
// in round w / 4), which go to the workspace as four partial rows per workgroup.  Sweep 2:
// dx = rstd (ghat - m1 - xhat m2) and its block max-abs; then quantize and store.
template <int B, int NIT>
__global__ void __launch_bounds__(1024) layernorm_bwd_wide_kernel(const int8_t* __restrict__ G, const float* __restrict__ SG,
                                                              const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                              const float* __restrict__ gamma,
                                                              const float* __restrict__ mean_in,
                                                              const float* __restrict__ rstd_in, int rows, int cols,
                                                              int8_t* __restrict__ dX, float* __restrict__ SdX,
                                                              float* __restrict__ partials) {
  constexpr int NW = 16, RW = B / NW;
  constexpr bool KEEP = RW * NIT <= 2;    // codes of x and g stay in registers
  constexpr bool KEEPY = RW * NIT <= 2;   // dx stays in registers between the max-abs and the quantize step
  extern __shared__ float s_dyn[];        // [NW][C/32] block max-abs, then [4][2][C] column sums
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r0 = blockIdx.x * B + wave * RW;
  const int lc = cols / B, bi = blockIdx.x, nchunks = cols / 16, ngran = cols / 32;
  float* s_amax = s_dyn;
  float* s_col = s_dyn + NW * ngran;

  bool ok[NIT];
  float sx[NIT], sg[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int c = lane + 64 * it;
    ok[it] = c < nchunks;
    sx[it] = ok[it] ? SX[(int64_t)bi * lc + (16 * c) / B] : 0.0f;
    sg[it] = ok[it] ? SG[(int64_t)bi * lc + (16 * c) / B] : 0.0f;
  }
  uint4 xs[KEEP ? RW : 1][NIT], gs[KEEP ? RW : 1][NIT];
  auto chunk_x = [&](int r, int it) -> uint4 {
    if (KEEP) return xs[r][it];
    return *reinterpret_cast<const uint4*>(X + (int64_t)(r0 + r) * cols + 16 * (lane + 64 * it));
  };
  auto chunk_g = [&](int r, int it) -> uint4 {
    if (KEEP) return gs[r][it];
    return *reinterpret_cast<const uint4*>(G + (int64_t)(r0 + r) * cols + 16 * (lane + 64 * it));
  };
  if (KEEP) {
#pragma unroll
    for (int r = 0; r < RW; ++r)
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int64_t off = (int64_t)(r0 + r) * cols + 16 * (lane + 64 * it);
        xs[r][it] = ok[it] ? *reinterpret_cast<const uint4*>(X + off) : make_uint4(0, 0, 0, 0);
        gs[r][it] = ok[it] ? *reinterpret_cast<const uint4*>(G + off) : make_uint4(0, 0, 0, 0);
      }
  }
  float mu[RW], rs[RW], m1[RW], m2[RW];
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    mu[r] = mean_in[r0 + r];
    rs[r] = rstd_in[r0 + r];
    m1[r] = m2[r] = 0.0f;
  }

  // sweep 1: row sums, and column sums folded over the waves in four rounds (per chunk column, so that only
  // one chunk's 32 column sums are live in registers)
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    float cg[16], cb[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) cg[e] = cb[e] = 0.0f;
    if (ok[it]) {
      float gm[16];
      load16f(gamma + 16 * (lane + 64 * it), gm);
      const float g128 = -128.0f * sg[it];
#pragma unroll
      for (int r = 0; r < RW; ++r) {
        float ux[16], ug[16];
        unpack16_biased(chunk_x(r, it), ux);
        unpack16_biased(chunk_g(r, it), ug);
        const float kx = sx[it] * rs[r], cx = __builtin_fmaf(-128.0f, kx, -mu[r] * rs[r]);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float xh = __builtin_fmaf(ux[e], kx, cx);
          const float gv = __builtin_fmaf(ug[e], sg[it], g128);
          const float gh = gv * gm[e];
          m1[r] += gh;
          m2[r] = __builtin_fmaf(gh, xh, m2[r]);
          cg[e] = __builtin_fmaf(gv, xh, cg[e]);
          cb[e] += gv;
        }
      }
    }
#pragma unroll
    for (int round = 0; round < 4; ++round) {
      if ((wave >> 2) == round && ok[it]) {
        float* row_g = s_col + (wave & 3) * 2 * cols + 16 * (lane + 64 * it);
        float* row_b = row_g + cols;
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          float4 a = make_float4(cg[4 * d], cg[4 * d + 1], cg[4 * d + 2], cg[4 * d + 3]);
          float4 b = make_float4(cb[4 * d], cb[4 * d + 1], cb[4 * d + 2], cb[4 * d + 3]);
          if (round > 0) {
            const float4 pa = *reinterpret_cast<const float4*>(row_g + 4 * d);
            const float4 pb = *reinterpret_cast<const float4*>(row_b + 4 * d);
            a = make_float4(pa.x + a.x, pa.y + a.y, pa.z + a.z, pa.w + a.w);
            b = make_float4(pb.x + b.x, pb.y + b.y, pb.z + b.z, pb.w + b.w);
          }
          *reinterpret_cast<float4*>(row_g + 4 * d) = a;
          *reinterpret_cast<float4*>(row_b + 4 * d) = b;
        }
      }
      __syncthreads();
    }
  }
  {  // the four folded rows -> workspace: thread t copies float4 number t, t + 1024, ...
    float* dst = partials + (int64_t)blockIdx.x * 4 * 2 * cols;
    for (int i = threadIdx.x; i < 4 * 2 * cols / 4; i += 1024)
      *reinterpret_cast<float4*>(dst + 4 * i) = *reinterpret_cast<const float4*>(s_col + 4 * i);
  }

  // dx = ug * a_c + ux * kxm + (a_c * -128 + krow) with a_c = rstd * sg * gamma_c
  float kxm[RW][NIT], krow[RW][NIT];
#pragma unroll
  for (int r = 0; r < RW; ++r) {
    const float q1 = wave_group_sum<63>(m1[r]) / (float)cols;
    const float q2 = wave_group_sum<63>(m2[r]) / (float)cols;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const float kx = sx[it] * rs[r], cx = __builtin_fmaf(-128.0f, kx, -mu[r] * rs[r]);
      kxm[r][it] = -rs[r] * q2 * kx;
      krow[r][it] = -rs[r] * __builtin_fmaf(cx, q2, q1);
    }
  }
  auto dx16 = [&](int r, int it, const float (&gm)[16], float (&y)[16]) {
    float ux[16], ug[16];
    unpack16_biased(chunk_x(r, it), ux);
    unpack16_biased(chunk_g(r, it), ug);
    const float rsg = rs[r] * sg[it];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const float a = rsg * gm[e];
      const float k = __builtin_fmaf(a, -128.0f, krow[r][it]);
      y[e] = __builtin_fmaf(ux[e], kxm[r][it], __builtin_fmaf(ug[e], a, k));
    }
  };

  // sweep 2
  constexpr int LM = B / 16 - 1;
  float ys[KEEPY ? RW : 1][KEEPY ? NIT : 1][16];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    float m = 0.0f;
    if (ok[it]) {
      float gm[16];
      load16f(gamma + 16 * (lane + 64 * it), gm);
#pragma unroll
      for (int r = 0; r < RW; ++r) {
        float y[16];
        dx16(r, it, gm, y);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          if (KEEPY) ys[r][it][e] = y[e];
          m = fmaxf(m, fabsf(y[e]));
        }
      }
    }
    m = wave_group_max<LM>(m);
    const int c = lane + 64 * it;
    if (ok[it] && (c & 1) == 0) s_amax[wave * ngran + (c >> 1)] = m;
  }
  __syncthreads();

  // quantize and store
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int c = lane + 64 * it;
    if (ok[it]) {
      float mm = 0.0f, scale;
      double inv;
#pragma unroll
      for (int w = 0; w < NW; ++w) mm = fmaxf(mm, s_amax[w * ngran + (c >> 1)]);
      block_scale(mm, scale, inv);
      if (wave == 0 && ((16 * c) % B) == 0) SdX[(int64_t)bi * lc + (16 * c) / B] = scale;
      if (KEEPY) {
#pragma unroll
        for (int r = 0; r < RW; ++r)
          *reinterpret_cast<uint4*>(dX + (int64_t)(r0 + r) * cols + 16 * c) = quantize16(ys[r][it], inv);
      } else {
        float gm[16];
        load16f(gamma + 16 * c, gm);
#pragma unroll
        for (int r = 0; r < RW; ++r) {
          float y[16];
          dx16(r, it, gm, y);
          *reinterpret_cast<uint4*>(dX + (int64_t)(r0 + r) * cols + 16 * c) = quantize16(y, inv);
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// LayerNorm at block size 32.  Where whole rows are needed a workgroup owns 32 of them and is made of strip waves:
// wave w holds the 32 x 128 strip w of those rows with the lane mapping of Strip32 (C / 128 waves, at most 16).  What
// needs a whole row (the row sums) is reduced over the 8 chunk lanes of a row inside each wave (three DPP steps)
// and over the strips through a few hundred bytes of LDS, in a fixed order; what belongs to a block (max-abs,
// scale) or to a column (gamma, beta, the column sums of the backward pass) never leaves its wave.
// WMAX = most waves the instance is compiled for (the register budget follows from it).
struct RowStrips32 {
  int ch, rsub, wave, nstrips;
  int lc, col;
  bool ok;
  __device__ __forceinline__ RowStrips32(int cols) {
    const int lane = threadIdx.x & 63;
    ch = lane & 7;
    rsub = lane >> 3;
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    nstrips = blockDim.x >> 6;
    lc = cols / 32;
    // rows wider than 16 strips are shared by the workgroups blockIdx.y = 0, 1, ...: 2048 columns each
    const int c0 = (blockIdx.y * 16 + wave) * 128, c = c0 + 16 * ch;
    ok = c < cols;
    col = ok ? c : min(c0, cols - 32);   // lanes outside the matrix point at a valid chunk instead, see Strip32
  }
  // element offset of the lane's chunk of row rsub of block row bi; pass p adds 8 p cols
  __device__ __forceinline__ int64_t base(int bi, int cols) const { return (int64_t)(bi * 32 + rsub) * cols + col; }
  __device__ __forceinline__ int64_t block_index(int bi) const { return (int64_t)bi * lc + col / 32; }
};

// Row statistics of LayerNorm from the codes (the per-row mean and sum of squares of App. A, here taken of the INT8 input
// itself), for rows of any width: the workgroup's waves share the strips of its 32 rows (wave w takes strips w, w + waves, ...).
// Per 16-code chunk the sum and the sum of squares of the codes are exact integers (v_dot4); times the block scale,
// in double, they are the chunk's share of the row's sum and sum of squares.  The shares are added over a lane's
// strips, over the 8 chunk lanes of a row (three DPP steps) and over the waves through LDS, in a fixed order.  The
// normalisation itself is layernorm_apply_strip32_kernel, an element-wise operator on strips.
__global__ void __launch_bounds__(1024) layernorm_row_stats_strips32_kernel(const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                                           float eps, int rows, int cols,
                                                                           float* __restrict__ mean_out, float* __restrict__ rstd_out) {
  __shared__ double s_row[16][32][2];
  const int lane = threadIdx.x & 63, ch = lane & 7, rsub = lane >> 3;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nwaves = blockDim.x >> 6;
  const int bi = blockIdx.x, lc = cols / 32;
  const int64_t pass = (int64_t)8 * cols;
  double cs[4] = {0.0, 0.0, 0.0, 0.0}, cq[4] = {0.0, 0.0, 0.0, 0.0};
  for (int c0 = wave * 128; c0 < cols; c0 += nwaves * 128) {
    const bool ok = c0 + 16 * ch < cols;
    const int col = ok ? c0 + 16 * ch : c0;   // lanes outside the matrix read the strip's first chunk and add nothing
    const int64_t base = (int64_t)(bi * 32 + rsub) * cols + col;
    uint4 px[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) px[p] = *reinterpret_cast<const uint4*>(X + base + p * pass);
    const double sd = ok ? (double)SX[(int64_t)bi * lc + col / 32] : 0.0;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      int s1, s2;
      chunk_moments(px[p], s1, s2);
      cs[p] += sd * (double)s1;
      cq[p] += sd * sd * (double)s2;
    }
  }
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const double s = wave_group_sum_f64<7>(cs[p]), q = wave_group_sum_f64<7>(cq[p]);
    if (ch == 0) {
      s_row[wave][rsub + 8 * p][0] = s;
      s_row[wave][rsub + 8 * p][1] = q;
    }
  }
  __syncthreads();
  if (threadIdx.x < 32) {   // row threadIdx.x of the block: the waves in a fixed order
    double s = 0.0, q = 0.0;
    for (int w = 0; w < nwaves; ++w) {
      s += s_row[w][threadIdx.x][0];
      q += s_row[w][threadIdx.x][1];
    }
    const double inv_cols = 1.0 / (double)cols, mud = s * inv_cols;
    const float var = fmaxf((float)(q * inv_cols - mud * mud), 0.0f);
    // reciprocal square root: hardware approximation refined by one Newton step (relative error ~1e-7)
    const float ve = var + eps;
    float rs = __builtin_amdgcn_rsqf(ve);
    rs = rs * __builtin_fmaf(-0.5f * ve * rs, rs, 1.5f);
    mean_out[bi * 32 + threadIdx.x] = (float)mud;
    rstd_out[bi * 32 + threadIdx.x] = rs;
  }
}

// LayerNorm backward at block size 32, in two kernels.  With ghat = g gamma and xhat = (x - mean) rstd,
//   dx = rstd (ghat - mean_C(ghat) - xhat mean_C(ghat xhat)),  dgamma = sum_N g xhat,  dbeta = sum_N g.
// Everything that needs a whole row or a whole column is a sum, and sums are cheap to hand over: the first kernel
// reads g and x once and leaves the two row means per row and one row of dgamma | dbeta partial sums per workgroup
// in the workspace; the second one is an element-wise operator on 32 x 128 strips like GELU backward.  (One kernel
// that does both has to keep dx, the codes and the column sums in registers at once: about 250, which leaves a
// compute unit with a single workgroup and nothing to overlap its memory latency with.)
//
// First kernel: the workgroup of strip waves described above walks over the row blocks blockIdx.x, blockIdx.x +
// gridDim.x, ... (four waves per SIMD: another workgroup's loads run beside this one's arithmetic).  The row sums go
// over the chunk lanes, then over the strips through LDS (two copies used by alternate row blocks: one barrier per block); the running column sums of
// g xhat and g stay in registers over all row blocks -- a lane always holds the same 16 columns -- and are added
// over the 8 row lanes of the wave at the end (every wave owns its own 128 columns of the partial row).  All orders
// are fixed: results are bit-stable from run to run.
template <int WMAX>
__global__ void __launch_bounds__(64 * WMAX) __attribute__((amdgpu_waves_per_eu(4))) layernorm_bwd_sums_strips32_kernel(
    const int8_t* __restrict__ G, const float* __restrict__ SG, const int8_t* __restrict__ X, const float* __restrict__ SX,
    const float* __restrict__ gamma, const float* __restrict__ mean_in, const float* __restrict__ rstd_in, int rows,
    int cols, float* __restrict__ row_means, float* __restrict__ partials) {
  __shared__ float s_row[2][WMAX][32][2];   // [row block parity][strip][row]: sums of ghat and of ghat xhat
  const RowStrips32 t(cols);
  const int64_t pass = (int64_t)8 * cols;
  const int nblocks = rows / 32;
  const float inv_cols = 1.0f / (float)cols;
  float gm[16], cgs[16], cbs[16];
  load16f(gamma + t.col, gm);
#pragma unroll
  for (int e = 0; e < 16; ++e) cgs[e] = cbs[e] = 0.0f;

  int parity = 0;
  for (int bi = blockIdx.x; bi < nblocks; bi += gridDim.x, parity ^= 1) {
    const int64_t base = t.base(bi, cols);
    uint4 px[4], pg[4];
    float mu[4], rs[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      px[p] = *reinterpret_cast<const uint4*>(X + base + p * pass);
      pg[p] = *reinterpret_cast<const uint4*>(G + base + p * pass);
      mu[p] = mean_in[bi * 32 + t.rsub + 8 * p];
      rs[p] = rstd_in[bi * 32 + t.rsub + 8 * p];
    }
    const float sx = SX[t.block_index(bi)];
    const float sg = t.ok ? SG[t.block_index(bi)] : 0.0f;   // lanes outside the matrix add nothing to the sums
    const float g128 = -128.0f * sg;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      float ux[16], ug[16];
      unpack16_biased(px[p], ux);
      unpack16_biased(pg[p], ug);
      const float kx = sx * rs[p], cx0 = __builtin_fmaf(-128.0f, kx, -mu[p] * rs[p]);
      float m1 = 0.0f, m2 = 0.0f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float xh = __builtin_fmaf(ux[e], kx, cx0);
        const float gv = __builtin_fmaf(ug[e], sg, g128);
        const float gh = gv * gm[e];
        m1 += gh;
        m2 = __builtin_fmaf(gh, xh, m2);
        // the column sums are updated in place, in program order (left to itself the compiler parks them in
        // scratch memory and keeps the operands of sixteen deferred updates alive instead)
        asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(cgs[e]) : "v"(gv), "v"(xh));
        asm volatile("v_add_f32 %0, %0, %1" : "+v"(cbs[e]) : "v"(gv));
      }
      m1 = wave_group_sum<7>(m1);
      m2 = wave_group_sum<7>(m2);
      if (t.ch == 0) {
        s_row[parity][t.wave][t.rsub + 8 * p][0] = m1;
        s_row[parity][t.wave][t.rsub + 8 * p][1] = m2;
      }
      __builtin_amdgcn_sched_barrier(0);   // one pass at a time: interleaved passes keep their unpacked values live together
    }
    __syncthreads();
    if (threadIdx.x < 32) {   // row threadIdx.x of the block: the strips in a fixed order
      float q1 = 0.0f, q2 = 0.0f;
      for (int w = 0; w < t.nstrips; ++w) {
        q1 += s_row[parity][w][threadIdx.x][0];
        q2 += s_row[parity][w][threadIdx.x][1];
      }
      // (the share of this workgroup's column range; the second kernel adds the ranges)
      *reinterpret_cast<float2*>(row_means + 2 * ((int64_t)blockIdx.y * rows + bi * 32 + threadIdx.x)) =
          make_float2(q1 * inv_cols, q2 * inv_cols);
    }
  }

  // column sums over the 8 row lanes of the wave; the lanes of row 0 write the wave's 128 columns of the partial row
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    cgs[e] = wave_group_sum<56>(cgs[e]);
    cbs[e] = wave_group_sum<56>(cbs[e]);
  }
  if (t.ok && t.rsub == 0) {
    float* dst = partials + (int64_t)blockIdx.x * 2 * cols + t.col;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      *reinterpret_cast<float4*>(dst + 4 * d) = make_float4(cgs[4 * d], cgs[4 * d + 1], cgs[4 * d + 2], cgs[4 * d + 3]);
      *reinterpret_cast<float4*>(dst + cols + 4 * d) = make_float4(cbs[4 * d], cbs[4 * d + 1], cbs[4 * d + 2], cbs[4 * d + 3]);
    }
  }
}

// Second kernel: dx on 32 x 128 strips, one wave each, from the row means q1 = mean_C(ghat), q2 = mean_C(ghat xhat)
// that the first kernel left (one share per range of 2048 columns): dx = ug a_c + ux b + d with per-row
// b = -rstd q2 sx rstd and d, and per-column a_c = rstd sg gamma_c (u = code + 128), then Eq. 1.  Rows may be of any
// width.
__global__ void __launch_bounds__(64 * kStripWaves) layernorm_bwd_apply_strip32_kernel(
    const int8_t* __restrict__ G, const float* __restrict__ SG, const int8_t* __restrict__ X, const float* __restrict__ SX,
    const float* __restrict__ gamma, const float* __restrict__ mean_in, const float* __restrict__ rstd_in,
    const float* __restrict__ row_means, int ranges, int rows, int cols, int8_t* __restrict__ dX, float* __restrict__ SdX) {
  const Strip32 t(rows, cols);
  if (!t.inside) return;   // a whole wave; the strip kernels have no workgroup barrier
  const int64_t pass = (int64_t)8 * cols;
  uint4 px[4], pg[4];
  float mu[4], rs[4];
  float2 q[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    px[p] = *reinterpret_cast<const uint4*>(X + t.base + p * pass);
    pg[p] = *reinterpret_cast<const uint4*>(G + t.base + p * pass);
    const int row = t.bi * 32 + t.rsub + 8 * p;
    mu[p] = mean_in[row];
    rs[p] = rstd_in[row];
    q[p] = *reinterpret_cast<const float2*>(row_means + 2 * (int64_t)row);
    for (int cr = 1; cr < ranges; ++cr) {   // rows wider than 2048 columns: the column ranges in a fixed order
      const float2 part = *reinterpret_cast<const float2*>(row_means + 2 * ((int64_t)cr * rows + row));
      q[p].x += part.x;
      q[p].y += part.y;
    }
  }
  const float sx = SX[t.block_index()], sg = SG[t.block_index()];
  float gm[16];
  load16f(gamma + (t.ok ? t.col : t.c0), gm);
  float y[4][16];
  float m = 0.0f;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    float ux[16], ug[16];
    unpack16_biased(px[p], ux);
    unpack16_biased(pg[p], ug);
    const float kx = sx * rs[p], cx0 = __builtin_fmaf(-128.0f, kx, -mu[p] * rs[p]);
    const float kxm = -rs[p] * q[p].y * kx, krow = -rs[p] * __builtin_fmaf(cx0, q[p].y, q[p].x);
    const float rsg = rs[p] * sg;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const float a = rsg * gm[e];
      const float k = __builtin_fmaf(a, -128.0f, krow);
      y[p][e] = __builtin_fmaf(ux[e], kxm, __builtin_fmaf(ug[e], a, k));
    }
    m = amax16(m, y[p]);
  }
  float scale;
  double inv;
  strip32_block_scale(m, scale, inv);
  if (!t.ok) return;
  if ((t.lane & 57) == 0) SdX[t.block_index()] = scale;
#pragma unroll
  for (int p = 0; p < 4; ++p) *reinterpret_cast<uint4*>(dX + t.base + p * pass) = quantize16(y[p], inv);
}

// Row statistics of LayerNorm from the row partials that the preceding Add wrote (App. A, LayerNorm paragraph):
//   mean_i = (1 / L_C) sum_j row_mean[i][j],  var_i = max((1 / C) sum_j row_sumsq[i][j] - mean_i^2, 0),
// summed in double in a fixed order; rstd as the hardware reciprocal square root plus one Newton step.  A group of
// 8 lanes owns a row: the lanes read the row's partials as consecutive floats (a wave reads eight rows, which lie
// back to back in memory) and add their shares with three butterfly steps.
__global__ void __launch_bounds__(256) row_stats_from_partials_kernel(const float* __restrict__ row_mean,
                                                                       const float* __restrict__ row_sumsq, float eps,
                                                                       int rows, int lc, int cols,
                                                                       float* __restrict__ mean_out, float* __restrict__ rstd_out) {
  const int sub = threadIdx.x & 7;
  const int row = min(blockIdx.x * 32 + (threadIdx.x >> 3), rows - 1);   // surplus groups repeat the last row
  const float* pm = row_mean + (int64_t)row * lc;
  const float* pq = row_sumsq + (int64_t)row * lc;
  double s = 0.0, q = 0.0;
  for (int j = sub; j < lc; j += 8) {
    s += (double)pm[j];
    q += (double)pq[j];
  }
  s = wave_group_sum_f64<7>(s);
  q = wave_group_sum_f64<7>(q);
  const double mu = s / (double)lc;
  const float var = fmaxf((float)(q / (double)cols - mu * mu), 0.0f);
  const float ve = var + eps;
  float rs = __builtin_amdgcn_rsqf(ve);
  rs = rs * __builtin_fmaf(-0.5f * ve * rs, rs, 1.5f);
  if (sub == 0) {
    mean_out[row] = (float)mu;
    rstd_out[row] = rs;
  }
}

// LayerNorm at block size 32 from given row statistics (App. A: the operator is handed the row mean and rstd):
// y = (x - mean) rstd gamma + beta on 32 x 128 strips, one wave each, like the other element-wise operators --
// no workgroup needs a whole row, so rows may be of any width.
__global__ void __launch_bounds__(64 * kStripWaves) layernorm_apply_strip32_kernel(const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                                     const float* __restrict__ gamma, const float* __restrict__ beta,
                                                                     const float* __restrict__ mean_in, const float* __restrict__ rstd_in,
                                                                     int rows, int cols, int8_t* __restrict__ Y, float* __restrict__ SY) {
  const Strip32 t(rows, cols);
  if (!t.inside) return;   // a whole wave; the strip kernels have no workgroup barrier
  const int64_t pass = (int64_t)8 * cols;
  uint4 px[4];
  float mu[4], rs[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    px[p] = *reinterpret_cast<const uint4*>(X + t.base + p * pass);
    mu[p] = mean_in[t.bi * 32 + t.rsub + 8 * p];
    rs[p] = rstd_in[t.bi * 32 + t.rsub + 8 * p];
  }
  const float sx = SX[t.block_index()];
  float gm[16], bt[16];
  const int gcol = t.ok ? t.col : t.c0;
  load16f(gamma + gcol, gm);
  load16f(beta + gcol, bt);
  float y[4][16];
  float m = 0.0f;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    float u[16];
    unpack16_biased(px[p], u);
    const float k1 = sx * rs[p], kb = __builtin_fmaf(-128.0f, k1, -mu[p] * rs[p]);
#pragma unroll
    for (int e = 0; e < 16; ++e) y[p][e] = __builtin_fmaf(__builtin_fmaf(u[e], k1, kb), gm[e], bt[e]);
    m = amax16(m, y[p]);
  }
  float scale;
  double inv;
  strip32_block_scale(m, scale, inv);
  if (!t.ok) return;
  if ((t.lane & 57) == 0) SY[t.block_index()] = scale;
#pragma unroll
  for (int p = 0; p < 4; ++p) *reinterpret_cast<uint4*>(Y + t.base + p * pass) = quantize16(y[p], inv);
}

// dgamma / dbeta: sum the per-wave partial rows in a fixed order (bit-stable from run to run).  A workgroup
// of 16 waves owns 64 columns of the 2*C wide partial matrix; wave w sums rows w, w+16, w+32, ... (eight
// independent chains keep loads in flight), and wave 0 adds the 16 results in wave order.
__global__ void __launch_bounds__(1024) colsum_kernel(const float* __restrict__ partials, int nparts, int cols2,
                                                       float* __restrict__ dgamma, float* __restrict__ dbeta) {
  __shared__ float s_part[16][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  float acc[8] = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
  if (c < cols2) {
    int p = wave;
    for (; p + 112 < nparts; p += 128) {
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = partials[(int64_t)(p + 16 * j) * cols2 + c];
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += v[j];
    }
    for (; p < nparts; p += 16) acc[0] += partials[(int64_t)p * cols2 + c];
  }
  s_part[wave][lane] = ((acc[0] + acc[1]) + (acc[2] + acc[3])) + ((acc[4] + acc[5]) + (acc[6] + acc[7]));
  __syncthreads();
  if (wave == 0 && c < cols2) {
    float v = 0.0f;
#pragma unroll
    for (int w = 0; w < 16; ++w) v += s_part[w][lane];
    const int half = cols2 / 2;
    if (c < half) dgamma[c] = v;
    else dbeta[c - half] = v;
  }
}

// ------------------------------------------------------------------------------------------------ host
// LayerNorm rows are held as NIT 16-byte chunks per lane; the register budget caps NIT at 4 (C <= 4096).
constexpr int64_t kLayerNormMaxC = 4096;

template <int B, int NIT, typename... Args>
static void launch_ln_fwd(bool from_partials, dim3 grid, size_t lds, hipStream_t st, Args... args) {
  if (from_partials) hipLaunchKernelGGL((layernorm_fwd_kernel<B, NIT, true>), grid, dim3(1024), lds, st, args...);
  else hipLaunchKernelGGL((layernorm_fwd_kernel<B, NIT, false>), grid, dim3(1024), lds, st, args...);
}
template <int B, int NIT, typename... Args>
static void launch_ln_bwd(dim3 grid, size_t lds, hipStream_t st, Args... args) {
  if constexpr (NIT <= 2) hipLaunchKernelGGL((layernorm_bwd_kernel<B, NIT>), grid, dim3(512), lds, st, args...);
  else hipLaunchKernelGGL((layernorm_bwd_wide_kernel<B, NIT>), grid, dim3(1024), lds, st, args...);
}

#define JF_LN_DISPATCH(FN, block, nit, ...)                                   \
  do {                                                                        \
    if (block == 32) {                                                        \
      if (nit == 1) FN<32, 1>(__VA_ARGS__);                                   \
      else if (nit == 2) FN<32, 2>(__VA_ARGS__);                              \
      else FN<32, 4>(__VA_ARGS__);                                            \
    } else if (block == 64) {                                                 \
      if (nit == 1) FN<64, 1>(__VA_ARGS__);                                   \
      else if (nit == 2) FN<64, 2>(__VA_ARGS__);                              \
      else FN<64, 4>(__VA_ARGS__);                                            \
    } else {                                                                  \
      if (nit == 1) FN<128, 1>(__VA_ARGS__);                                  \
      else if (nit == 2) FN<128, 2>(__VA_ARGS__);                             \
      else FN<128, 4>(__VA_ARGS__);                                           \
    }                                                                         \
  } while (0)

}  // namespace jf

template <typename... Args>
static void launch_ln_bwd_sums_strips32(int64_t C, dim3 grid, hipStream_t st, Args... args) {
  const int ns = (int)std::min<int64_t>(16, (C + 127) / 128);   // waves; the last column range may use fewer of them
  if (ns <= 4) hipLaunchKernelGGL((jf::layernorm_bwd_sums_strips32_kernel<4>), grid, dim3(64 * ns), 0, st, args...);
  else if (ns <= 8) hipLaunchKernelGGL((jf::layernorm_bwd_sums_strips32_kernel<8>), grid, dim3(64 * ns), 0, st, args...);
  else hipLaunchKernelGGL((jf::layernorm_bwd_sums_strips32_kernel<16>), grid, dim3(64 * ns), 0, st, args...);
}

static int32_t layernorm_fwd(const int8_t* X, const float* SX, const float* row_mean, const float* row_sumsq,
                             const float* gamma, const float* beta, float eps, int64_t N, int64_t C, int32_t block,
                             int8_t* Y, float* SY, float* mean, float* rstd, void* stream) {
  using namespace jf;
  int32_t rc = check_eltwise(X, SX, Y, SY, N, C, block);
  if (rc != JF_OK) return rc;
  if (!gamma || !beta || !mean || !rstd) return JF_ERR_NULL;
  // Block size 32: a statistics kernel (from the Add's partials, or from the codes) and the normalisation on
  // 32 x 128 strips; no workgroup holds a whole row in registers, so rows may be of any width.
  const bool strips = block == 32;
  if (C > kLayerNormMaxC && !strips) return JF_ERR_SHAPE;
  if (!aligned16(gamma) || !aligned16(beta) || !aligned4(mean) || !aligned4(rstd)) return JF_ERR_ALIGN;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (strips) {
    if (row_mean != nullptr) {
      hipLaunchKernelGGL(row_stats_from_partials_kernel, dim3((unsigned)((N + 31) / 32)), dim3(256), 0, st, row_mean, row_sumsq,
                         eps, (int)N, (int)(C / 32), (int)C, mean, rstd);
    } else {
      const int waves = (int)std::min<int64_t>(16, (C + 127) / 128);
      hipLaunchKernelGGL(layernorm_row_stats_strips32_kernel, dim3((unsigned)(N / 32)), dim3(64 * waves), 0, st, X, SX, eps, (int)N,
                         (int)C, mean, rstd);
    }
    rc = launch_status();
    if (rc != JF_OK) return rc;
    hipLaunchKernelGGL(layernorm_apply_strip32_kernel, strip_grid(N, C), dim3(64 * kStripWaves), 0, st, X, SX, gamma,
                       beta, mean, rstd, (int)N, (int)C, Y, SY);
    return launch_status();
  }
  const dim3 grid((unsigned)(N / block));
  const int nit = (int)((C + 1023) / 1024);
  const size_t lds = 16 * (size_t)(C / 32) * sizeof(float);
  JF_LN_DISPATCH(launch_ln_fwd, block, nit, row_mean != nullptr, grid, lds, st, X, SX, gamma, beta, eps, (int)N, (int)C, Y, SY, mean, rstd,
                 row_mean, row_sumsq);
  return launch_status();
}

extern "C" int32_t jf_layernorm_q(const int8_t* X, const float* SX, const float* gamma, const float* beta, float eps,
                                  int64_t N, int64_t C, int32_t block, int8_t* Y, float* SY, float* mean, float* rstd,
                                  void* stream) {
  return layernorm_fwd(X, SX, nullptr, nullptr, gamma, beta, eps, N, C, block, Y, SY, mean, rstd, stream);
}

extern "C" int32_t jf_layernorm_q_partials(const int8_t* X, const float* SX, const float* row_mean,
                                           const float* row_sumsq, const float* gamma, const float* beta, float eps,
                                           int64_t N, int64_t C, int32_t block, int8_t* Y, float* SY, float* mean,
                                           float* rstd, void* stream) {
  if (!row_mean || !row_sumsq) return JF_ERR_NULL;
  if (!jf::aligned4(row_mean) || !jf::aligned4(row_sumsq)) return JF_ERR_ALIGN;
  return layernorm_fwd(X, SX, row_mean, row_sumsq, gamma, beta, eps, N, C, block, Y, SY, mean, rstd, stream);
}

// LayerNorm backward behind both entry points: `partials` is the caller's workspace or this library's static
// scratch; every argument has been validated.
static int32_t layernorm_bwd_launch(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX,
                                    const float* gamma, const float* mean, const float* rstd, int64_t N, int64_t C,
                                    int32_t block, int8_t* dX, float* SdX, float* dgamma, float* dbeta, float* partials,
                                    hipStream_t st) {
  using namespace jf;
  const int nparts = (int)ln_bwd_partial_rows(N, C, block);
  const dim3 grid((unsigned)(C > 2048 ? N / block : nparts));
  if (block == 32) {
    // the workspace holds the partial rows, then the two row means of every row (per range of 2048 columns)
    float* row_means = partials + (size_t)nparts * 2 * (size_t)C;
    const int ranges = (int)((C + 2047) / 2048);
    launch_ln_bwd_sums_strips32(C, dim3((unsigned)nparts, (unsigned)ranges), st, dY, SdY, X, SX, gamma, mean, rstd, (int)N, (int)C,
                                row_means, partials);
    const int32_t rc1 = launch_status();
    if (rc1 != JF_OK) return rc1;
    hipLaunchKernelGGL(layernorm_bwd_apply_strip32_kernel, strip_grid(N, C), dim3(64 * kStripWaves), 0, st, dY, SdY, X, SX,
                       gamma, mean, rstd, row_means, ranges, (int)N, (int)C, dX, SdX);
  } else {
    const int nit = (int)((C + 1023) / 1024);
    // max-abs slots per wave, (row means,) four column-sum rows
    const size_t lds = C > 2048 ? (16 * (size_t)(C / 32) + 4 * 2 * (size_t)C) * sizeof(float)
                                : (8 * (size_t)(C / 32) + 2 * (size_t)block + 4 * 2 * (size_t)C) * sizeof(float);
    JF_LN_DISPATCH(launch_ln_bwd, block, nit, grid, lds, st, dY, SdY, X, SX, gamma, mean, rstd, (int)N, (int)C, dX, SdX, partials);
  }
  const int32_t rc = launch_status();
  if (rc != JF_OK) return rc;
  hipLaunchKernelGGL(colsum_kernel, dim3((unsigned)((2 * C + 63) / 64)), dim3(1024), 0, st, partials, nparts, (int)(2 * C), dgamma, dbeta);
  return launch_status();
}

static int32_t layernorm_bwd_check(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX,
                                   const float* gamma, const float* mean, const float* rstd, int64_t N, int64_t C,
                                   int32_t block, int8_t* dX, float* SdX, float* dgamma, float* dbeta) {
  using namespace jf;
  int32_t rc = check_eltwise(X, SX, dX, SdX, N, C, block);
  if (rc != JF_OK) return rc;
  if (!dY || !SdY || !gamma || !mean || !rstd || !dgamma || !dbeta) return JF_ERR_NULL;
  if (C > kLayerNormMaxC && block != 32) return JF_ERR_SHAPE;
  if (!aligned16(dY) || !aligned4(SdY) || !aligned16(gamma) || !aligned4(mean) || !aligned4(rstd) ||
      !aligned4(dgamma) || !aligned4(dbeta))
    return JF_ERR_ALIGN;
  return JF_OK;
}

extern "C" int32_t jf_layernorm_q_bwd(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX,
                                      const float* gamma, const float* mean, const float* rstd, int64_t N, int64_t C,
                                      int32_t block, int8_t* dX, float* SdX, float* dgamma, float* dbeta, void* ws,
                                      size_t ws_bytes, void* stream) {
  int32_t rc = layernorm_bwd_check(dY, SdY, X, SX, gamma, mean, rstd, N, C, block, dX, SdX, dgamma, dbeta);
  if (rc != JF_OK) return rc;
  const size_t need = jf_workspace_bytes(JF_OP_LAYERNORM_BWD, N, C, 0, block);
  if (!ws || ws_bytes < need) return JF_ERR_WORKSPACE;
  if (!jf::aligned16(ws)) return JF_ERR_ALIGN;
  return layernorm_bwd_launch(dY, SdY, X, SX, gamma, mean, rstd, N, C, block, dX, SdX, dgamma, dbeta,
                              static_cast<float*>(ws), reinterpret_cast<hipStream_t>(stream));
}

// ------------------------------------------------------------------------------------------------
// The entry point that allocates nothing: jf_layernorm_q_bwd with its workspace (the partial rows of
// dgamma | dbeta) in a static device array instead of a caller-provided buffer.  In host code the array's
// name is only a handle: its device address is looked up once per device, with that device current, and that
// pointer is what the kernels receive.  Every GPU holds its own copy of the array until the process ends.
static __device__ __align__(256) unsigned char scratch[JF_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, once looked up

// Device address of the static scratch on the current device (nullptr and *rc = JF_ERR_LAUNCH on failure).
void* static_scratch(int32_t* rc) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess && (dev < 0 || dev >= kMaxDevices)) e = hipErrorInvalidDevice;
  if (e == hipSuccess) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e == hipSuccess && p == nullptr) e = hipErrorInvalidSymbol;
      if (e == hipSuccess) g_scratch_ptr[dev] = p;
    }
    if (e == hipSuccess) return g_scratch_ptr[dev];
  }
  jf::g_last_hip_error = (int32_t)e;
  *rc = JF_ERR_LAUNCH;
  return nullptr;
}
}  // namespace

extern "C" int32_t jf_layernorm_q_bwd_static(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX,
                                             const float* gamma, const float* mean, const float* rstd, int64_t N,
                                             int64_t C, int32_t block, int8_t* dX, float* SdX, float* dgamma,
                                             float* dbeta, void* stream) {
  int32_t rc = layernorm_bwd_check(dY, SdY, X, SX, gamma, mean, rstd, N, C, block, dX, SdX, dgamma, dbeta);
  if (rc != JF_OK) return rc;
  if (jf_workspace_bytes(JF_OP_LAYERNORM_BWD, N, C, 0, block) > (size_t)JF_STATIC_SCRATCH_BYTES) return JF_ERR_WORKSPACE;
  void* const ptr = static_scratch(&rc);
  if (ptr == nullptr) return rc;
  // Nothing in the scratch has to start at zero: every partial row that the second kernel reads is written
  // in full by the first one of the same call.
  return layernorm_bwd_launch(dY, SdY, X, SX, gamma, mean, rstd, N, C, block, dX, SdX, dgamma, dbeta,
                              static_cast<float*>(ptr), reinterpret_cast<hipStream_t>(stream));
}
