// INT8-in / INT8-out LayerNorm, forward and backward (App. A).
//
// Each pass is a small kernel that only leaves sums (row statistics forward; row means and dgamma | dbeta partial rows
// backward) followed by an element-wise operator on tiles: the 32 x 128 strips of jf_rowops.hpp at block size 32, workgroups
// of B rows x 128 columns at block sizes 64 and 128.  No workgroup holds a row in registers, so rows may be of any width.
// Row sums of the forward pass come from exact integer dot products of the codes (v_dot4), scaled per block -- the
// row-partials scheme of App. A applied to the INT8 input itself -- or from the partials that the preceding Add wrote.
#include <algorithm>
#include <mutex>

#include "jf_rowops.hpp"

namespace jf {

// ------------------------------------------------------------------------------------------------
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

// ------------------------------------------------------------------------------------------------
// Where whole rows are needed a workgroup owns 32 of them (at every block size: a block row is one, two or four such
// groups) and is made of strip waves: wave w holds the 32 x 128 strip w of those rows with the lane mapping of Strip32
// (C / 128 waves, at most 16).  What
// needs a whole row (the row sums) is reduced over the 8 chunk lanes of a row inside each wave (three DPP steps)
// and over the strips through a few hundred bytes of LDS, in a fixed order; what belongs to a block (max-abs,
// scale) or to a column (gamma, beta, the column sums of the backward pass) never leaves its wave.
// WMAX = most waves the instance is compiled for (the register budget follows from it).
struct RowStrips {
  int ch, rsub, wave, nstrips;
  int lc, col, block;
  bool ok;
  __device__ __forceinline__ RowStrips(int cols, int block_size) {
    const int lane = threadIdx.x & 63;
    ch = lane & 7;
    rsub = lane >> 3;
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    nstrips = blockDim.x >> 6;
    block = block_size;
    lc = cols / block;
    // rows wider than 16 strips are shared by the workgroups blockIdx.y = 0, 1, ...: 2048 columns each
    const int c0 = (blockIdx.y * 16 + wave) * 128, c = c0 + 16 * ch;
    ok = c < cols;
    col = ok ? c : min(c0, cols - 32);   // lanes outside the matrix point at a valid chunk instead, see Strip32
  }
  // element offset of the lane's chunk of row rsub of the 32-row group g; pass p adds 8 p cols
  __device__ __forceinline__ int64_t base(int g, int cols) const { return (int64_t)(g * 32 + rsub) * cols + col; }
  // index of the lane's quantization block in a scale grid
  __device__ __forceinline__ int64_t block_index(int g) const { return (int64_t)(g * 32 / block) * lc + col / block; }
};

// Row statistics of LayerNorm from the codes (the per-row mean and sum of squares of App. A, here taken of the INT8 input
// itself), for rows of any width: the workgroup's waves share the strips of its 32 rows (wave w takes strips w, w + waves, ...).
// Per 16-code chunk the sum and the sum of squares of the codes are exact integers (v_dot4); times the block scale,
// in double, they are the chunk's share of the row's sum and sum of squares.  The shares are added over a lane's
// strips, over the 8 chunk lanes of a row (three DPP steps) and over the waves through LDS, in a fixed order.  The
// normalisation itself is layernorm_apply_strip32_kernel, an element-wise operator on strips.
__global__ void __launch_bounds__(1024) layernorm_row_stats_kernel(const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                                  float eps, int rows, int cols, int block,
                                                                           float* __restrict__ mean_out, float* __restrict__ rstd_out) {
  __shared__ double s_row[16][32][2];
  const int lane = threadIdx.x & 63, ch = lane & 7, rsub = lane >> 3;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nwaves = blockDim.x >> 6;
  const int bi = blockIdx.x, lc = cols / block;   // bi: group of 32 rows
  const int64_t pass = (int64_t)8 * cols;
  double cs[4] = {0.0, 0.0, 0.0, 0.0}, cq[4] = {0.0, 0.0, 0.0, 0.0};
  for (int c0 = wave * 128; c0 < cols; c0 += nwaves * 128) {
    const bool ok = c0 + 16 * ch < cols;
    const int col = ok ? c0 + 16 * ch : c0;   // lanes outside the matrix read the strip's first chunk and add nothing
    const int64_t base = (int64_t)(bi * 32 + rsub) * cols + col;
    uint4 px[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) px[p] = *reinterpret_cast<const uint4*>(X + base + p * pass);
    const double sd = ok ? (double)SX[(int64_t)(bi * 32 / block) * lc + col / block] : 0.0;
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

// LayerNorm backward, in two kernels.  With ghat = g gamma and xhat = (x - mean) rstd,
//   dx = rstd (ghat - mean_C(ghat) - xhat mean_C(ghat xhat)),  dgamma = sum_N g xhat,  dbeta = sum_N g.
// Everything that needs a whole row or a whole column is a sum, and sums are cheap to hand over: the first kernel
// reads g and x once and leaves the two row means per row and one row of dgamma | dbeta partial sums per workgroup
// in the workspace; the second one is an element-wise operator on tiles like GELU backward.  (One kernel
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
__global__ void __launch_bounds__(64 * WMAX) __attribute__((amdgpu_waves_per_eu(4))) layernorm_bwd_sums_kernel(
    const int8_t* __restrict__ G, const float* __restrict__ SG, const int8_t* __restrict__ X, const float* __restrict__ SX,
    const float* __restrict__ gamma, const float* __restrict__ mean_in, const float* __restrict__ rstd_in, int rows,
    int cols, int block, float* __restrict__ row_means, float* __restrict__ partials) {
  __shared__ float s_row[2][WMAX][32][2];   // [row block parity][strip][row]: sums of ghat and of ghat xhat
  const RowStrips t(cols, block);
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
//   mean_i = (1 / L_C) sum_j row_mean[j][i],  var_i = max((1 / C) sum_j row_sumsq[j][i] - mean_i^2, 0),
// summed in double in a fixed order; rstd as the hardware reciprocal square root plus one Newton step.  The partials are
// stored block-column-major ((C / B) x N): a workgroup owns 64 consecutive rows, lane = row, so every load of a wave is
// 64 consecutive floats; its waves (4 to 16, about one per four block columns) take the block columns j = w, w + waves,
// ... and their shares are added through LDS in wave order.
__global__ void __launch_bounds__(1024) row_stats_from_partials_kernel(const float* __restrict__ row_mean,
                                                                        const float* __restrict__ row_sumsq, float eps,
                                                                        int rows, int lc, int cols,
                                                                        float* __restrict__ mean_out, float* __restrict__ rstd_out) {
  __shared__ double s_part[16][64][2];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, NW = blockDim.x >> 6;
  const int row = min((int)blockIdx.x * 64 + lane, rows - 1);   // lanes past the last row repeat it and write nothing
  double s = 0.0, q = 0.0;
  for (int j = wave; j < lc; j += NW) {
    s += (double)row_mean[(int64_t)j * rows + row];
    q += (double)row_sumsq[(int64_t)j * rows + row];
  }
  s_part[wave][lane][0] = s;
  s_part[wave][lane][1] = q;
  __syncthreads();
  if (wave != 0 || (int)blockIdx.x * 64 + lane >= rows) return;
  s = q = 0.0;
  for (int w = 0; w < NW; ++w) {
    s += s_part[w][lane][0];
    q += s_part[w][lane][1];
  }
  const double mu = s / (double)lc;
  const float var = fmaxf((float)(q / (double)cols - mu * mu), 0.0f);
  const float ve = var + eps;
  float rs = __builtin_amdgcn_rsqf(ve);
  rs = rs * __builtin_fmaf(-0.5f * ve * rs, rs, 1.5f);
  mean_out[row] = (float)mu;
  rstd_out[row] = rs;
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

// The same two element-wise operators at block sizes 64 and 128: one workgroup of four waves owns B rows x 128 columns
// (two blocks resp. one); wave w owns rows [w B/4, (w+1) B/4) in B/32 passes of 8 rows with the lane mapping of the
// strips (lane = (row l / 8, 16-byte chunk l % 8): full 128-byte lines); the block max-abs goes over the lanes of a
// block column inside a wave and over the four waves through LDS.  MODE 0: y = (x - mean) rstd gamma + beta (forward),
// MODE 1: dx from the row means of the sums kernel (backward).
template <int B, int MODE>
__global__ void __launch_bounds__(256) layernorm_tile_kernel(const int8_t* __restrict__ G, const float* __restrict__ SG,
                                                              const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                              const float* __restrict__ gamma, const float* __restrict__ beta,
                                                              const float* __restrict__ mean_in, const float* __restrict__ rstd_in,
                                                              const float* __restrict__ row_means, int ranges, int rows, int cols,
                                                              int8_t* __restrict__ Y, float* __restrict__ SY) {
  constexpr int P = B / 32;
  __shared__ float s_amax[4][4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ch = lane & 7, rsub = lane >> 3;
  const TileIndex wg = tile_of_workgroup((cols + 127) / 128);
  const int col = wg.x * 128 + 16 * ch;
  const int r0 = wg.y * B + wave * (B / 4);
  const bool col_ok = col < cols;
  const int lc = cols / B, bi = wg.y;

  float y[P][16];
  float m = 0.0f;
  if (col_ok) {
    const float sx = SX[(int64_t)bi * lc + col / B];
    float gm[16], bt[16];
    load16f(gamma + col, gm);
    float sg = 0.0f;
    if (MODE == 0) load16f(beta + col, bt);
    else sg = SG[(int64_t)bi * lc + col / B];
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int row = r0 + 8 * p + rsub;
      const float mu = mean_in[row], rs = rstd_in[row];
      float ux[16];
      unpack16_biased(*reinterpret_cast<const uint4*>(X + (int64_t)row * cols + col), ux);
      const float kx = sx * rs, cx0 = __builtin_fmaf(-128.0f, kx, -mu * rs);   // xhat = ux kx + cx0, ux = code + 128
      if (MODE == 0) {
#pragma unroll
        for (int e = 0; e < 16; ++e) y[p][e] = __builtin_fmaf(__builtin_fmaf(ux[e], kx, cx0), gm[e], bt[e]);
      } else {
        float2 q = *reinterpret_cast<const float2*>(row_means + 2 * (int64_t)row);
        for (int cr = 1; cr < ranges; ++cr) {   // rows wider than 2048 columns: the column ranges in a fixed order
          const float2 part = *reinterpret_cast<const float2*>(row_means + 2 * ((int64_t)cr * rows + row));
          q.x += part.x;
          q.y += part.y;
        }
        float ug[16];
        unpack16_biased(*reinterpret_cast<const uint4*>(G + (int64_t)row * cols + col), ug);
        const float kxm = -rs * q.y * kx, krow = -rs * __builtin_fmaf(cx0, q.y, q.x), rsg = rs * sg;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float a = rsg * gm[e];
          y[p][e] = __builtin_fmaf(ux[e], kxm, __builtin_fmaf(ug[e], a, __builtin_fmaf(a, -128.0f, krow)));
        }
      }
      m = amax16(m, y[p]);
    }
  }
  m = strip_block_max<B>(m);
  // s_amax[wave][32-column group]; the in-wave reduction already covered the whole block width
  if ((lane & 57) == 0) s_amax[wave][ch >> 1] = m;
  __syncthreads();
  m = fmaxf(fmaxf(s_amax[0][ch >> 1], s_amax[1][ch >> 1]), fmaxf(s_amax[2][ch >> 1], s_amax[3][ch >> 1]));
  float scale;
  double inv;
  block_scale(m, scale, inv);
  if (!col_ok) return;
  if (wave == 0 && rsub == 0 && (col % B) == 0) SY[(int64_t)bi * lc + col / B] = scale;
#pragma unroll
  for (int p = 0; p < P; ++p) {
    const int row = r0 + 8 * p + rsub;
    *reinterpret_cast<uint4*>(Y + (int64_t)row * cols + col) = quantize16(y[p], inv);
  }
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
}  // namespace jf

template <typename... Args>
static void launch_ln_bwd_sums(int64_t C, dim3 grid, hipStream_t st, Args... args) {
  const int ns = (int)std::min<int64_t>(16, (C + 127) / 128);   // waves; the last column range may use fewer of them
  if (ns <= 4) hipLaunchKernelGGL((jf::layernorm_bwd_sums_kernel<4>), grid, dim3(64 * ns), 0, st, args...);
  else if (ns <= 8) hipLaunchKernelGGL((jf::layernorm_bwd_sums_kernel<8>), grid, dim3(64 * ns), 0, st, args...);
  else hipLaunchKernelGGL((jf::layernorm_bwd_sums_kernel<16>), grid, dim3(64 * ns), 0, st, args...);
}

// A statistics kernel (from the Add's partials, or from the codes), then the normalisation on tiles.
static int32_t layernorm_fwd(const int8_t* X, const float* SX, const float* row_mean, const float* row_sumsq,
                             const float* gamma, const float* beta, float eps, int64_t N, int64_t C, int32_t block,
                             int8_t* Y, float* SY, float* mean, float* rstd, void* stream) {
  using namespace jf;
  int32_t rc = check_eltwise(X, SX, Y, SY, N, C, block);
  if (rc != JF_OK) return rc;
  if (!gamma || !beta || !mean || !rstd) return JF_ERR_NULL;
  if (!aligned16(gamma) || !aligned16(beta) || !aligned4(mean) || !aligned4(rstd)) return JF_ERR_ALIGN;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (row_mean != nullptr) {
    const int waves = (int)std::min<int64_t>(16, std::max<int64_t>(4, C / block / 4));
    hipLaunchKernelGGL(row_stats_from_partials_kernel, dim3((unsigned)((N + 63) / 64)), dim3(64 * waves), 0, st, row_mean, row_sumsq,
                       eps, (int)N, (int)(C / block), (int)C, mean, rstd);
  } else {
    const int waves = (int)std::min<int64_t>(16, (C + 127) / 128);
    hipLaunchKernelGGL(layernorm_row_stats_kernel, dim3((unsigned)(N / 32)), dim3(64 * waves), 0, st, X, SX, eps, (int)N, (int)C,
                       (int)block, mean, rstd);
  }
  rc = launch_status();
  if (rc != JF_OK) return rc;
  const dim3 tiles(tile_grid((C + 127) / 128, N / block));
  const float* none = nullptr;
  if (block == 32)
    hipLaunchKernelGGL(layernorm_apply_strip32_kernel, strip_grid(N, C), dim3(64 * kStripWaves), 0, st, X, SX, gamma, beta, mean,
                       rstd, (int)N, (int)C, Y, SY);
  else if (block == 64)
    hipLaunchKernelGGL((layernorm_tile_kernel<64, 0>), tiles, dim3(256), 0, st, (const int8_t*)nullptr, none, X, SX, gamma, beta,
                       (const float*)mean, (const float*)rstd, none, 1, (int)N, (int)C, Y, SY);
  else
    hipLaunchKernelGGL((layernorm_tile_kernel<128, 0>), tiles, dim3(256), 0, st, (const int8_t*)nullptr, none, X, SX, gamma, beta,
                       (const float*)mean, (const float*)rstd, none, 1, (int)N, (int)C, Y, SY);
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
  const int nparts = (int)ln_bwd_partial_rows(N);
  // the workspace holds the partial rows, then the two row means of every row (per range of 2048 columns)
  float* row_means = partials + (size_t)nparts * 2 * (size_t)C;
  const int ranges = (int)((C + 2047) / 2048);
  launch_ln_bwd_sums(C, dim3((unsigned)nparts, (unsigned)ranges), st, dY, SdY, X, SX, gamma, mean, rstd, (int)N, (int)C, (int)block,
                     row_means, partials);
  const int32_t rc1 = launch_status();
  if (rc1 != JF_OK) return rc1;
  const dim3 tiles(tile_grid((C + 127) / 128, N / block));
  const float* none = nullptr;
  if (block == 32)
    hipLaunchKernelGGL(layernorm_bwd_apply_strip32_kernel, strip_grid(N, C), dim3(64 * kStripWaves), 0, st, dY, SdY, X, SX, gamma,
                       mean, rstd, row_means, ranges, (int)N, (int)C, dX, SdX);
  else if (block == 64)
    hipLaunchKernelGGL((layernorm_tile_kernel<64, 1>), tiles, dim3(256), 0, st, dY, SdY, X, SX, gamma, none, mean, rstd,
                       (const float*)row_means, ranges, (int)N, (int)C, dX, SdX);
  else
    hipLaunchKernelGGL((layernorm_tile_kernel<128, 1>), tiles, dim3(256), 0, st, dY, SdY, X, SX, gamma, none, mean, rstd,
                       (const float*)row_means, ranges, (int)N, (int)C, dX, SdX);
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
