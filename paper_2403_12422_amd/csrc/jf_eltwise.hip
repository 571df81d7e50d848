// INT8-in / INT8-out GELU (forward and backward), Add and Dropout (Sec. 6, Alg. 2, App. A).
//
// These kernels move 2-3 bytes per element, so at HBM speed a SIMD has 50-60 cycles per element, of which Eq. 1's exact
// rounding takes 14.  What keeps them inside that budget:
//   * GELU: within one quantization block the input takes at most 255 values (code * block scale), so GELU (or its
//     derivative) is tabulated once per block in LDS and every element is a table lookup indexed by its code byte -- the
//     dequantize step of Alg. 2 and the erf evaluation collapse into it;
//   * block size 32: one wave per strip of 32 x 128 (four blocks), 64 elements of one block per lane, no barrier, see
//     jf_rowops.hpp; block sizes 64 and 128 use workgroups of B rows x 128 or 256 columns.
#include "jf_rowops.hpp"

namespace jf {

// ------------------------------------------------------------------------------------------------
// One table of GELU (or its derivative) at the 255 values code * sx of a block, indexed by the code byte taken as
// unsigned: lane l evaluates codes l and l + 64 and, by symmetry, -l and -(l + 64).  Both functions are written in
// terms of the upper tail Q(a) = Phi(-a), a >= 0 (App. A):
//   GELU(x) = x Phi(x):  f(a) = a - a Q(a),  f(-a) = -a Q(a);
//   GELU'(x) = Phi(x) + x phi(x):  f(a) = 1 - Q(a) + a phi(a),  f(-a) = Q(a) - a phi(a),  phi(a) = exp(-a^2/2) / sqrt(2 pi).
//   Q(a) = t P(t) exp(-a^2/2),  t = 1 / (1 + a / sqrt(8)),  P of degree 8 fitted by weighted least squares on Chebyshev
//   nodes to erfcx(a / sqrt 2) / (2 t) for 0 <= a <= 13.4 (relative error 5e-8; evaluated in FP32: 4e-7).
// exp(-a^2/2) = 2^H (1 + r ln 2) with H = fl(-a^2 log2(e)/2) and r the exact remainder (product residuals by FMA),
// so that the FP32 rounding of an exponent of size a^2 does not cost log2(a^2) bits: Q keeps a relative error of
// about 1e-6 into the far tail, where a block that lies entirely there takes its scale from.
template <bool BWD>
__device__ __forceinline__ void gelu_table_entries(float a, float& pos, float& neg) {
  const float ac = fminf(a, 40.0f);                       // Q(40) = 0 in FP32; keeps a^2 finite
  const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(ac, 0.35355339059327373f, 1.0f));
  float p = -2.9970746985e-02f;
  p = __builtin_fmaf(p, t, 1.4432375881e-01f);
  p = __builtin_fmaf(p, t, -2.4760739076e-01f);
  p = __builtin_fmaf(p, t, 1.4335782902e-01f);
  p = __builtin_fmaf(p, t, -1.6097390692e-02f);
  p = __builtin_fmaf(p, t, 1.0243339323e-01f);
  p = __builtin_fmaf(p, t, 1.2129997806e-01f);
  p = __builtin_fmaf(p, t, 1.4121892641e-01f);
  p = __builtin_fmaf(p, t, 1.4104161820e-01f);
  const float K = -0.72134752044448170f;                  // -log2(e) / 2
  const float aa = ac * ac;
  const float lo = __builtin_fmaf(ac, ac, -aa);           // a^2 = aa + lo exactly
  const float H = aa * K;
  const float r = __builtin_fmaf(lo, K, __builtin_fmaf(aa, K, -H));
  const float ez = __builtin_amdgcn_exp2f(H) * __builtin_fmaf(r, 0.6931471805599453f, 1.0f);   // exp(-a^2/2)
  const float q = (t * p) * ez;
  if (BWD) {
    const float s = (a * 0.39894228040143268f) * ez;      // a phi(a)
    pos = (1.0f - q) + s;
    neg = q - s;
  } else {
    const float aq = a * q;
    pos = a - aq;
    neg = 0.0f - aq;
  }
}

template <bool BWD>
__device__ __forceinline__ void gelu_build_table(float* tab, float sx, int lane) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int i = lane + 64 * h;
    float pos, neg;
    gelu_table_entries<BWD>((float)i * sx, pos, neg);
    // code 0: GELU(0) = 0 comes out exactly; GELU'(0) = 1/2 is set, because the fit is only good to 4e-7 there and a
    // derivative of 0.49999997 would push every halved gradient code off its rounding tie.  Entry 128 (code -128,
    // which no quantizer output holds) is 0.
    tab[i] = (BWD && i == 0) ? 0.5f : pos;
    tab[i == 0 ? 128 : 256 - i] = i == 0 ? 0.0f : neg;
  }
}

// ------------------------------------------------------------------------------------------------
// GELU forward / backward at block sizes 64 and 128 (large tensors at 64).  One workgroup of four waves owns B rows x J*128 columns = J*128/min(B,128)
// quantization blocks; wave w owns rows [w*B/4, (w+1)*B/4) in B/32 passes of 8 rows, lane = (row l/8,
// 16-byte chunk l%8) in each of the J 128-column halves, so every row segment is a full 128-byte line.
// J = 2 (B = 64) halves the number of workgroups; the tables built per element stay the same.
template <bool BWD, int B, int J>
__global__ void __launch_bounds__(256) gelu_kernel(const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                    const int8_t* __restrict__ G, const float* __restrict__ SG,
                                                    int rows, int cols, int8_t* __restrict__ Y, float* __restrict__ SY) {
  constexpr int P = B / 32;                  // 8-row passes per wave
  constexpr int TPH = B >= 128 ? 1 : 128 / B;  // quantization blocks (= tables) per 128-column half
  constexpr int NTAB = J * TPH;
  __shared__ float s_tab[NTAB][256];         // indexed by the code byte taken as unsigned
  __shared__ float s_amax[4][4 * J];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ch = lane & 7, rsub = lane >> 3;
  const TileIndex wg = tile_of_workgroup((cols + 128 * J - 1) / (128 * J));
  const int c0 = wg.x * (128 * J);
  const int r0 = wg.y * B + wave * (B / 4);
  const int lc = cols / B, bi = wg.y;
  int col[J];
  bool col_ok[J];  // cols % 32 == 0 and chunks are 16 wide: a 32-column group is all in or all out
#pragma unroll
  for (int j = 0; j < J; ++j) {
    col[j] = c0 + 128 * j + 16 * ch;
    col_ok[j] = col[j] < cols;
  }

  // The workgroup's codes are requested first: their latency runs beside the table build below.
  uint4 px[J][P], pg[J][BWD ? P : 1];
#pragma unroll
  for (int j = 0; j < J; ++j) {
    if (col_ok[j]) {
#pragma unroll
      for (int p = 0; p < P; ++p) {
        const int64_t off = (int64_t)(r0 + 8 * p + rsub) * cols + col[j];
        px[j][p] = *reinterpret_cast<const uint4*>(X + off);
        if (BWD) pg[j][p] = *reinterpret_cast<const uint4*>(G + off);
      }
    }
  }

  // Tabulate f(code * scale) for the byte values of each block of this workgroup.  Both functions are
  // built from the upper tail Q(|x|), so one tail evaluation serves the codes +i and -i: 128 evaluations
  // per table.  Entry 128 (code -128, which no quantizer output holds) is set to 0.
  {
    const int i = threadIdx.x & 127;
    // the table index is the same for all lanes of a wave, so the block scale comes through the scalar cache
    // (constant address space: the grid is never written by this kernel)
    typedef const __attribute__((address_space(4))) float* const_f32_ptr;
    const const_f32_ptr sx_row = (const_f32_ptr)SX + (int64_t)bi * lc;
#pragma unroll
    for (int k = __builtin_amdgcn_readfirstlane(threadIdx.x >> 7); k < NTAB; k += 2) {
      const int bcol = c0 + (k / TPH) * 128 + (k % TPH) * B;
      if (bcol < cols) {
        float pos, neg;  // f(+a), f(-a)
        gelu_table_entries<BWD>((float)i * sx_row[bcol / B], pos, neg);
        // code 0: GELU'(0) = 1/2 exactly, entry 128 unused: see gelu_build_table
        s_tab[k][i] = (BWD && i == 0) ? 0.5f : pos;
        s_tab[k][i == 0 ? 128 : 256 - i] = i == 0 ? 0.0f : neg;
      }
    }
  }
  __syncthreads();

  float y[J][P][16];
#pragma unroll
  for (int j = 0; j < J; ++j) {
    float m = 0.0f;
    if (col_ok[j]) {
      const float* tab = s_tab[j * TPH + (16 * ch) / B];
      float sg = 0.0f, sg128 = 0.0f;
      if (BWD) {
        sg = SG[(int64_t)bi * lc + col[j] / B];
        sg128 = -128.0f * sg;
      }
#pragma unroll
      for (int p = 0; p < P; ++p) {
        const uint32_t w[4] = {px[j][p].x, px[j][p].y, px[j][p].z, px[j][p].w};
        float f[16];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          f[4 * d + 0] = tab[w[d] & 0xffu];
          f[4 * d + 1] = tab[(w[d] >> 8) & 0xffu];
          f[4 * d + 2] = tab[(w[d] >> 16) & 0xffu];
          f[4 * d + 3] = tab[w[d] >> 24];
        }
        if (BWD) {
          float ug[16];
          unpack16_biased(pg[j][p], ug);
#pragma unroll
          for (int e = 0; e < 16; ++e) y[j][p][e] = __builtin_fmaf(ug[e], sg, sg128) * f[e];
        } else {
#pragma unroll
          for (int e = 0; e < 16; ++e) y[j][p][e] = f[e];
        }
#pragma unroll
        for (int e = 0; e < 16; e += 4) m = amax4(m, y[j][p][e], y[j][p][e + 1], y[j][p][e + 2], y[j][p][e + 3]);
      }
    }
    m = strip_block_max<B>(m);
    // s_amax[wave][32-column group]; for B >= 64 the in-wave reduction already covered the whole block width
    if ((lane & 57) == 0) s_amax[wave][4 * j + (ch >> 1)] = m;
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int gi = 4 * j + (ch >> 1);
    const float m = fmaxf(fmaxf(s_amax[0][gi], s_amax[1][gi]), fmaxf(s_amax[2][gi], s_amax[3][gi]));
    float scale;
    double inv;
    block_scale(m, scale, inv);
    if (!col_ok[j]) continue;
    if (wave == 0 && rsub == 0 && (col[j] % B) == 0) SY[(int64_t)bi * lc + col[j] / B] = scale;
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int row = r0 + 8 * p + rsub;
      *reinterpret_cast<uint4*>(Y + (int64_t)row * cols + col[j]) = quantize16(y[j][p], inv);
    }
  }
}

// GELU forward / backward for B = 64 (tensors that the last-level cache holds) with one quantization block per WAVE: the wave builds the block's
// table, looks its B x B codes up, takes the block max-abs with a wave reduction and stores -- no workgroup
// barrier and no LDS exchange between waves, so the four waves of a workgroup (four neighbouring block columns)
// run independently and one wave's table build overlaps its neighbours' loads and stores.  Lane = (row l / CPR,
// 16-byte chunk l % CPR) with CPR = B/16 chunks per block row, in B*CPR/64 passes; the four waves of a workgroup
// read neighbouring 32- or 64-byte pieces of the same memory lines.
template <bool BWD, int B>
__global__ void __launch_bounds__(256) gelu_wave_kernel(const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                         const int8_t* __restrict__ G, const float* __restrict__ SG,
                                                         int rows, int cols, int8_t* __restrict__ Y, float* __restrict__ SY) {
  constexpr int CPR = B / 16, RPP = 64 / CPR, P = B / RPP;  // chunks per block row, rows per pass, passes
  __shared__ float s_tab[4][256];  // one table per wave, indexed by the code byte taken as unsigned
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lc = cols / B;
  const TileIndex wg = tile_of_workgroup((lc + 3) / 4);
  const int bi = wg.y, bj = wg.x * 4 + wave;
  if (bj >= lc) return;  // wave-uniform; the kernel has no workgroup barrier
  const int ch = lane % CPR, rsub = lane / CPR;
  const int64_t base = (int64_t)(bi * B + rsub) * cols + bj * B + 16 * ch;

  // codes first: their latency runs beside the table build
  uint4 px[P], pg[BWD ? P : 1];
#pragma unroll
  for (int p = 0; p < P; ++p) {
    px[p] = *reinterpret_cast<const uint4*>(X + base + (int64_t)p * RPP * cols);
    if (BWD) pg[p] = *reinterpret_cast<const uint4*>(G + base + (int64_t)p * RPP * cols);
  }

  // the block's table: 128 tail evaluations, two per lane (see gelu_kernel); scales through the scalar cache
  typedef const __attribute__((address_space(4))) float* const_f32_ptr;
  const float sx = ((const_f32_ptr)SX)[(int64_t)bi * lc + bj];
  float* tab = s_tab[wave];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int i = lane + 64 * h;
    float pos, neg;
    gelu_table_entries<BWD>((float)i * sx, pos, neg);
    tab[i] = (BWD && i == 0) ? 0.5f : pos;  // GELU'(0) = 1/2 exactly, see gelu_build_table
    tab[i == 0 ? 128 : 256 - i] = i == 0 ? 0.0f : neg;
  }
  // The table is written and read by this wave only; LDS serves a wave's accesses in program order, and the
  // fence keeps the compiler from moving the lookups above the writes.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  float sg = 0.0f, sg128 = 0.0f;
  if (BWD) {
    sg = ((const_f32_ptr)SG)[(int64_t)bi * lc + bj];
    sg128 = -128.0f * sg;
  }
  float y[P][16];
  float m = 0.0f;
#pragma unroll
  for (int p = 0; p < P; ++p) {
    const uint32_t w[4] = {px[p].x, px[p].y, px[p].z, px[p].w};
    float f[16];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      f[4 * d + 0] = tab[w[d] & 0xffu];
      f[4 * d + 1] = tab[(w[d] >> 8) & 0xffu];
      f[4 * d + 2] = tab[(w[d] >> 16) & 0xffu];
      f[4 * d + 3] = tab[w[d] >> 24];
    }
    if (BWD) {
      float ug[16];
      unpack16_biased(pg[p], ug);
#pragma unroll
      for (int e = 0; e < 16; ++e) y[p][e] = __builtin_fmaf(ug[e], sg, sg128) * f[e];
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) y[p][e] = f[e];
    }
#pragma unroll
    for (int e = 0; e < 16; e += 4) m = amax4(m, y[p][e], y[p][e + 1], y[p][e + 2], y[p][e + 3]);
  }
  m = wave_group_max<63>(m);
  float scale;
  double inv;
  block_scale(m, scale, inv);
  if (lane == 0) SY[(int64_t)bi * lc + bj] = scale;
#pragma unroll
  for (int p = 0; p < P; ++p) *reinterpret_cast<uint4*>(Y + base + (int64_t)p * RPP * cols) = quantize16(y[p], inv);
}

// ------------------------------------------------------------------------------------------------
// Add (App. A): y = x1 + x2 on the dequantized operands, re-quantized per block (Alg. 2), and optionally
// the row partials that App. A's LayerNorm paragraph attaches to this operator: for every row and block
// column, the mean and the sum of squares of y over the block's B columns (stored block-column-major).  Same tiling as GELU.
template <int B>
__global__ void __launch_bounds__(256) add_kernel(const int8_t* __restrict__ X1, const float* __restrict__ S1,
                                                   const int8_t* __restrict__ X2, const float* __restrict__ S2, int rows,
                                                   int cols, int8_t* __restrict__ Y, float* __restrict__ SY,
                                                   float* __restrict__ row_mean, float* __restrict__ row_sumsq) {
  constexpr int P = B / 32;
  constexpr int CH = B >= 128 ? 7 : (B == 64 ? 3 : 1);  // chunk lanes of one block column
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
    const float s1 = S1[(int64_t)bi * lc + col / B], s2 = S2[(int64_t)bi * lc + col / B];
    const float k = -128.0f * (s1 + s2);  // the unpacked codes carry +128
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int row = r0 + 8 * p + rsub;
      float u1[16], u2[16];
      unpack16_biased(*reinterpret_cast<const uint4*>(X1 + (int64_t)row * cols + col), u1);
      unpack16_biased(*reinterpret_cast<const uint4*>(X2 + (int64_t)row * cols + col), u2);
      float ps = 0.0f, pq = 0.0f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        y[p][e] = __builtin_fmaf(u1[e], s1, __builtin_fmaf(u2[e], s2, k));
        ps += y[p][e];
        pq = __builtin_fmaf(y[p][e], y[p][e], pq);
      }
#pragma unroll
      for (int e = 0; e < 16; e += 4) m = amax4(m, y[p][e], y[p][e + 1], y[p][e + 2], y[p][e + 3]);
      if (row_mean != nullptr) {  // uniform over the grid
        ps = wave_group_sum<CH>(ps);
        pq = wave_group_sum<CH>(pq);
        if ((ch & CH) == 0) {
          row_mean[(int64_t)(col / B) * rows + row] = ps * (1.0f / (float)B);   // block-column-major, see jf_add_q
          row_sumsq[(int64_t)(col / B) * rows + row] = pq;
        }
      }
    }
  }
  m = strip_block_max<B>(m);
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

// ------------------------------------------------------------------------------------------------
// Dropout (App. A): y = x o m / (1 - p) on the dequantized input, re-quantized per block; the keep mask m is
// an input, packed 8 columns per byte (bit c % 8 of byte c / 8 of a row).  The backward pass is the same
// operator on the upstream gradient.  Same tiling as GELU; a lane's 16 columns are two mask bytes.
template <int B>
__global__ void __launch_bounds__(256) dropout_kernel(const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                       const uint8_t* __restrict__ mask, float keep_scale, int rows,
                                                       int cols, int8_t* __restrict__ Y, float* __restrict__ SY) {
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
    const float k = SX[(int64_t)bi * lc + col / B] * keep_scale;
    const float k128 = -128.0f * k;  // the unpacked codes carry +128
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int row = r0 + 8 * p + rsub;
      float u[16];
      unpack16_biased(*reinterpret_cast<const uint4*>(X + (int64_t)row * cols + col), u);
      const uint32_t bits = *reinterpret_cast<const uint16_t*>(mask + (int64_t)row * (cols / 8) + col / 8);
#pragma unroll
      for (int e = 0; e < 16; ++e) y[p][e] = ((bits >> e) & 1u) ? __builtin_fmaf(u[e], k, k128) : 0.0f;
#pragma unroll
      for (int e = 0; e < 16; e += 4) m = amax4(m, y[p][e], y[p][e + 1], y[p][e + 2], y[p][e + 3]);
    }
  }
  m = strip_block_max<B>(m);
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

// ------------------------------------------------------------------------------------------------
template <bool BWD>
__global__ void __launch_bounds__(64 * kStripWaves) gelu_strip32_kernel(const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                          const int8_t* __restrict__ G, const float* __restrict__ SG,
                                                          int rows, int cols, int8_t* __restrict__ Y, float* __restrict__ SY) {
  __shared__ float s_tabs[kStripWaves][4][256];
  float (*const s_tab)[256] = s_tabs[threadIdx.x >> 6];
  const Strip32 t(rows, cols);
  if (!t.inside) return;   // a whole wave; the strip kernels have no workgroup barrier
  const int64_t pass = (int64_t)8 * cols;
  // the codes are requested first: their latency runs beside the table build
  uint4 px[4], pg[BWD ? 4 : 1];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    px[p] = *reinterpret_cast<const uint4*>(X + t.base + p * pass);
    if (BWD) pg[p] = *reinterpret_cast<const uint4*>(G + t.base + p * pass);
  }
  // the strip's block scales are the same for all lanes: scalar loads (the grids are not written by this kernel)
  typedef const __attribute__((address_space(4))) float* const_f32_ptr;
  const const_f32_ptr sx_row = (const_f32_ptr)SX + (int64_t)t.bi * t.lc + t.c0 / 32;
  const int nblk = min(4, t.lc - t.c0 / 32);
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (k < nblk) gelu_build_table<BWD>(s_tab[k], sx_row[k], threadIdx.x & 63);
  // The tables are written and read by this wave only; LDS serves a wave's accesses in program order, and the
  // fences keep the compiler from moving the lookups above the writes.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  float y[4][16];
  float m = 0.0f;
  const float* tab = s_tab[t.ch >> 1];   // lanes outside the matrix may read a table nobody built: see Strip32::base
  float sg = 0.0f, sg128 = 0.0f;
  if (BWD) {
    sg = SG[t.block_index()];
    sg128 = -128.0f * sg;
  }
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const uint32_t w[4] = {px[p].x, px[p].y, px[p].z, px[p].w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      y[p][4 * d + 0] = tab[w[d] & 0xffu];
      y[p][4 * d + 1] = tab[(w[d] >> 8) & 0xffu];
      y[p][4 * d + 2] = tab[(w[d] >> 16) & 0xffu];
      y[p][4 * d + 3] = tab[w[d] >> 24];
    }
    if (BWD) {
      float ug[16];
      unpack16_biased(pg[p], ug);
#pragma unroll
      for (int e = 0; e < 16; ++e) y[p][e] = __builtin_fmaf(ug[e], sg, sg128) * y[p][e];
    }
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

// Add (App. A) at block size 32, optionally with the row partials of App. A's LayerNorm paragraph (PARTIALS).
template <bool PARTIALS>
__global__ void __launch_bounds__(64 * kStripWaves) add_strip32_kernel(const int8_t* __restrict__ X1, const float* __restrict__ S1,
                                                         const int8_t* __restrict__ X2, const float* __restrict__ S2,
                                                         int rows, int cols, int8_t* __restrict__ Y, float* __restrict__ SY,
                                                         float* __restrict__ row_mean, float* __restrict__ row_sumsq) {
  const Strip32 t(rows, cols);
  if (!t.inside) return;   // a whole wave; the strip kernels have no workgroup barrier
  const int64_t pass = (int64_t)8 * cols;
  float y[4][16];
  float m = 0.0f;
  uint4 p1[4], p2[4];
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    p1[p] = *reinterpret_cast<const uint4*>(X1 + t.base + p * pass);
    p2[p] = *reinterpret_cast<const uint4*>(X2 + t.base + p * pass);
  }
  const float s1 = S1[t.block_index()], s2 = S2[t.block_index()];
  const float k = -128.0f * (s1 + s2);  // the unpacked codes carry +128
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    float u1[16], u2[16];
    unpack16_biased(p1[p], u1);
    unpack16_biased(p2[p], u2);
#pragma unroll
    for (int e = 0; e < 16; ++e) y[p][e] = __builtin_fmaf(u1[e], s1, __builtin_fmaf(u2[e], s2, k));
    m = amax16(m, y[p]);
    if (PARTIALS) {  // per row and block: mean and sum of squares over the block's 32 columns = two neighbouring lanes
      float ps = 0.0f, pq = 0.0f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        ps += y[p][e];
        pq = __builtin_fmaf(y[p][e], y[p][e], pq);
      }
      ps = wave_group_sum<1>(ps);
      pq = wave_group_sum<1>(pq);
      if (t.ok && (t.ch & 1) == 0) {
        // block-column-major: the 32 rows of the strip are one 128-byte line per block column
        const int64_t o = (int64_t)(t.col / 32) * rows + (t.bi * 32 + t.rsub + 8 * p);
        row_mean[o] = ps * (1.0f / 32.0f);
        row_sumsq[o] = pq;
      }
    }
  }
  float scale;
  double inv;
  strip32_block_scale(m, scale, inv);
  if (!t.ok) return;
  if ((t.lane & 57) == 0) SY[t.block_index()] = scale;
#pragma unroll
  for (int p = 0; p < 4; ++p) *reinterpret_cast<uint4*>(Y + t.base + p * pass) = quantize16(y[p], inv);
}

// The four keep bits of one packed dword of codes -> 0xff / 0x00 per byte: the multiplication puts bit j of the
// nibble at bit 8 j (and copies elsewhere, which the mask removes), times 255 fills the byte.
__device__ __forceinline__ uint32_t keep_bytes(uint32_t nibble) {
  const uint32_t ones = (nibble * 0x00204081u) & 0x01010101u;
  uint32_t full;  // ones * 255 as shift and subtract (the compiler would make it a slow 32-bit multiplication)
  asm("v_lshlrev_b32 %0, 8, %1\n\tv_sub_u32 %0, %0, %1" : "=&v"(full) : "v"(ones));
  return full;
}

// Dropout (App. A) at block size 32: dropped codes are cleared in the packed dwords (a code of 0 dequantizes to
// exactly 0), so the mask costs a few integer instructions per four elements and none per element.
__global__ void __launch_bounds__(64 * kStripWaves) dropout_strip32_kernel(const int8_t* __restrict__ X, const float* __restrict__ SX,
                                                             const uint8_t* __restrict__ mask, float keep_scale, int rows,
                                                             int cols, int8_t* __restrict__ Y, float* __restrict__ SY) {
  const Strip32 t(rows, cols);
  if (!t.inside) return;   // a whole wave; the strip kernels have no workgroup barrier
  const int64_t pass = (int64_t)8 * cols;
  float y[4][16];
  float m = 0.0f;
  uint4 px[4];
  uint32_t bits[4];
  const int64_t mbase = t.base >> 3;   // row * (cols / 8) + column / 8: cols is a multiple of 32, the column of 16
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    px[p] = *reinterpret_cast<const uint4*>(X + t.base + p * pass);
    bits[p] = *reinterpret_cast<const uint16_t*>(mask + mbase + (int64_t)p * cols);   // 8 rows further: 8 * cols / 8 bytes
  }
  const float k = SX[t.block_index()] * keep_scale;
  const float k128 = -128.0f * k;  // the unpacked codes carry +128
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    uint4 c = px[p];
    c.x &= keep_bytes(bits[p] & 15u);
    c.y &= keep_bytes((bits[p] >> 4) & 15u);
    c.z &= keep_bytes((bits[p] >> 8) & 15u);
    c.w &= keep_bytes(bits[p] >> 12);
    float u[16];
    unpack16_biased(c, u);
#pragma unroll
    for (int e = 0; e < 16; ++e) y[p][e] = __builtin_fmaf(u[e], k, k128);
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

// ------------------------------------------------------------------------------------------------ host
template <bool BWD, int B>
static void launch_gelu_wave(const int8_t* X, const float* SX, const int8_t* G, const float* SG, int rows, int cols,
                             int8_t* Y, float* SY, hipStream_t st) {
  hipLaunchKernelGGL((gelu_wave_kernel<BWD, B>), dim3(tile_grid((cols / B + 3) / 4, rows / B)), dim3(256), 0, st, X, SX, G, SG,
                     rows, cols, Y, SY);
}
template <bool BWD, int B, int J>
static void launch_gelu_cfg(const int8_t* X, const float* SX, const int8_t* G, const float* SG, int rows, int cols,
                            int8_t* Y, float* SY, hipStream_t st) {
  hipLaunchKernelGGL((gelu_kernel<BWD, B, J>), dim3(tile_grid((cols + 128 * J - 1) / (128 * J), rows / B)), dim3(256), 0, st,
                     X, SX, G, SG, rows, cols, Y, SY);
}
template <bool BWD>
static void launch_gelu(int block, const int8_t* X, const float* SX, const int8_t* G, const float* SG, int rows,
                        int cols, int8_t* Y, float* SY, hipStream_t st) {
  // B = 32: one wave per workgroup and strip of 32 x 128 at every size.  B = 64: one block per wave while the
  // tensors are small enough to sit in the last-level cache (its 64-byte row pieces cost a third of the
  // bandwidth once the data comes from HBM: crossover near 100 M elements), beyond that one block per workgroup
  // column, in workgroups of 256 columns.  At B = 128 a lane already holds four 8-row passes of a 128-column workgroup.
  const int64_t n = (int64_t)rows * cols;
  if (block == 128) launch_gelu_cfg<BWD, 128, 1>(X, SX, G, SG, rows, cols, Y, SY, st);
  else if (block == 64) {
    if (n <= (int64_t(64) << 20)) launch_gelu_wave<BWD, 64>(X, SX, G, SG, rows, cols, Y, SY, st);
    else launch_gelu_cfg<BWD, 64, 2>(X, SX, G, SG, rows, cols, Y, SY, st);
  } else {
    hipLaunchKernelGGL((gelu_strip32_kernel<BWD>), strip_grid(rows, cols), dim3(64 * kStripWaves), 0, st, X, SX, G, SG,
                       rows, cols, Y, SY);
  }
}

}  // namespace jf

extern "C" int32_t jf_gelu_q(const int8_t* X, const float* SX, int64_t N, int64_t C, int32_t block, int8_t* Y,
                             float* SY, void* stream) {
  using namespace jf;
  int32_t rc = check_eltwise(X, SX, Y, SY, N, C, block);
  if (rc != JF_OK) return rc;
  launch_gelu<false>(block, X, SX, nullptr, nullptr, (int)N, (int)C, Y, SY, reinterpret_cast<hipStream_t>(stream));
  return launch_status();
}

extern "C" int32_t jf_gelu_q_bwd(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX, int64_t N,
                                 int64_t C, int32_t block, int8_t* dX, float* SdX, void* stream) {
  using namespace jf;
  int32_t rc = check_eltwise(X, SX, dX, SdX, N, C, block);
  if (rc != JF_OK) return rc;
  if (!dY || !SdY) return JF_ERR_NULL;
  if (!aligned16(dY) || !aligned4(SdY)) return JF_ERR_ALIGN;
  launch_gelu<true>(block, X, SX, dY, SdY, (int)N, (int)C, dX, SdX, reinterpret_cast<hipStream_t>(stream));
  return launch_status();
}

extern "C" int32_t jf_dropout_q(const int8_t* X, const float* SX, const uint8_t* mask_bits, float p, int64_t N, int64_t C,
                                int32_t block, int8_t* Y, float* SY, void* stream) {
  using namespace jf;
  int32_t rc = check_eltwise(X, SX, Y, SY, N, C, block);
  if (rc != JF_OK) return rc;
  if (!mask_bits) return JF_ERR_NULL;
  if (!(p >= 0.0f && p < 1.0f)) return JF_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(mask_bits) & 1u) return JF_ERR_ALIGN;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const dim3 grid(tile_grid((C + 127) / 128, N / block));
  const float keep_scale = (float)(1.0 / (1.0 - (double)p));
  const int rows = (int)N, cols = (int)C;
  if (block == 32)
    hipLaunchKernelGGL(dropout_strip32_kernel, strip_grid(N, C), dim3(64 * kStripWaves), 0, st, X, SX, mask_bits,
                       keep_scale, rows, cols, Y, SY);
  else if (block == 64) hipLaunchKernelGGL((dropout_kernel<64>), grid, dim3(256), 0, st, X, SX, mask_bits, keep_scale, rows, cols, Y, SY);
  else hipLaunchKernelGGL((dropout_kernel<128>), grid, dim3(256), 0, st, X, SX, mask_bits, keep_scale, rows, cols, Y, SY);
  return launch_status();
}

extern "C" int32_t jf_add_q(const int8_t* X1, const float* S1, const int8_t* X2, const float* S2, int64_t N, int64_t C,
                            int32_t block, int8_t* Y, float* SY, float* row_mean, float* row_sumsq, void* stream) {
  using namespace jf;
  int32_t rc = check_eltwise(X1, S1, Y, SY, N, C, block);
  if (rc != JF_OK) return rc;
  if (!X2 || !S2) return JF_ERR_NULL;
  if ((row_mean == nullptr) != (row_sumsq == nullptr)) return JF_ERR_NULL;
  if (!aligned16(X2) || !aligned4(S2) || (row_mean && (!aligned4(row_mean) || !aligned4(row_sumsq)))) return JF_ERR_ALIGN;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const dim3 grid(tile_grid((C + 127) / 128, N / block));
  const int rows = (int)N, cols = (int)C;
  if (block == 32) {
    const dim3 strips = strip_grid(N, C);
    if (row_mean) hipLaunchKernelGGL((add_strip32_kernel<true>), strips, dim3(64 * kStripWaves), 0, st, X1, S1, X2, S2, rows, cols, Y, SY, row_mean, row_sumsq);
    else hipLaunchKernelGGL((add_strip32_kernel<false>), strips, dim3(64 * kStripWaves), 0, st, X1, S1, X2, S2, rows, cols, Y, SY, row_mean, row_sumsq);
  } else if (block == 64) hipLaunchKernelGGL((add_kernel<64>), grid, dim3(256), 0, st, X1, S1, X2, S2, rows, cols, Y, SY, row_mean, row_sumsq);
  else hipLaunchKernelGGL((add_kernel<128>), grid, dim3(256), 0, st, X1, S1, X2, S2, rows, cols, Y, SY, row_mean, row_sumsq);
  return launch_status();
}
