// jf_quantize_block: per-block quantizer Q of Sec. 4, Eq. 1 (FP32/FP16 -> INT8 + FP32 scale grid).
//
// HBM-bound: 4 (or 2) bytes in, 1 byte out per element.  One workgroup of four
// waves owns a 128 x 128 tile; wave w owns the 32-row strip w of it.  Inside a
// strip a lane holds 4 consecutive columns of 16 rows, so each row of the strip
// is read as one 512-byte (FP32) run and written as one 128-byte run of codes.
#include "jf_common.hpp"

namespace jf {

template <typename T>
struct Load4;
template <>
struct Load4<float> {
  static __device__ __forceinline__ void run(const float* p, float (&v)[4]) {
    float4 t = *reinterpret_cast<const float4*>(p);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
  }
};
template <>
struct Load4<_Float16> {
  static __device__ __forceinline__ void run(const _Float16* p, float (&v)[4]) {
    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
    h4 t = *reinterpret_cast<const h4*>(p);
    v[0] = (float)t[0]; v[1] = (float)t[1]; v[2] = (float)t[2]; v[3] = (float)t[3];
  }
};

// B = quantization block; the tile is 128 x 128 and 256 threads (WPW = 4 waves per workgroup), or, for small
// tensors at B = 32 where the waves do not depend on each other, one 32 x 128 strip and one wave (WPW = 1), which
// spreads a tensor of a few hundred tiles over all compute units.
template <typename T, int B, bool TRANSPOSED_COPY, int WPW = 4>
__global__ void __launch_bounds__(64 * WPW) quantize_kernel(const T* __restrict__ x, int64_t ldx, int rows, int cols,
                                                        int8_t* __restrict__ q, int64_t ldq, float* __restrict__ s,
                                                        int8_t* __restrict__ qT, int64_t ldqT, float* __restrict__ sT) {
  __shared__ float s_amax[4][4];                       // [32-row strip][32-col group]
  __shared__ __align__(16) uint8_t s_codes[TRANSPOSED_COPY ? 128 * 132 : 16];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const TileIndex wg = tile_of_workgroup((cols + 127) / 128);
  static_assert(WPW == 4 || (WPW == 1 && B == 32 && !TRANSPOSED_COPY), "single-wave workgroups: independent waves only");
  const int r0 = (wg.y * WPW + wave) * 32;             // first row of this wave's strip
  const int c0 = wg.x * 128;
  const int c4 = lane & 31, rh = lane >> 5;
  const int col = c0 + 4 * c4;
  const bool col_ok = col < cols;                      // cols % 32 == 0: whole 8-lane groups are in or out

  float v[16][4];
  float amax = 0.0f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int row = r0 + 2 * i + rh;
    if (col_ok && row < rows) {
      Load4<T>::run(x + (int64_t)row * ldx + col, v[i]);
    } else {
      v[i][0] = v[i][1] = v[i][2] = v[i][3] = 0.0f;
    }
    amax = fmaxf(amax, fmaxf(fmaxf(fabsf(v[i][0]), fabsf(v[i][1])), fmaxf(fabsf(v[i][2]), fabsf(v[i][3]))));
  }
  // lanes sharing a 32-column group: same c4 / 8, any c4 % 8, any rh
  amax = wave_group_max<1 | 2 | 4 | 32>(amax);
  if (B > 32) {  // at B = 32 a block lies inside one wave's strip: no exchange, the waves run independently
    if ((lane & 39) == 0) s_amax[wave][c4 >> 3] = amax;
    __syncthreads();
    constexpr int G = B / 32;  // 32-granules per block side
    const int w0 = (wave / G) * G, g0 = ((c4 >> 3) / G) * G;
    amax = 0.0f;
#pragma unroll
    for (int a = 0; a < G; ++a)
#pragma unroll
      for (int b = 0; b < G; ++b) amax = fmaxf(amax, s_amax[w0 + a][g0 + b]);
  }
  float scale;
  double inv;
  block_scale(amax, scale, inv);

  const int lr = rows / B, lc = cols / B;
  // one lane per block writes the scale: the top-left 32-granule of the block
  if ((lane & 39) == 0 && col_ok && r0 < rows && (r0 % B) == 0 && ((c0 + 32 * (c4 >> 3)) % B) == 0) {
    const int bi = r0 / B, bj = (c0 + 32 * (c4 >> 3)) / B;
    s[(int64_t)bi * lc + bj] = scale;
    if (TRANSPOSED_COPY) sT[(int64_t)bj * lr + bi] = scale;
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int row = r0 + 2 * i + rh;
    const uint32_t packed = quantize4(v[i][0], v[i][1], v[i][2], v[i][3], inv);
    if (col_ok && row < rows) *reinterpret_cast<uint32_t*>(q + (int64_t)row * ldq + col) = packed;
    if (TRANSPOSED_COPY) *reinterpret_cast<uint32_t*>(&s_codes[(wave * 32 + 2 * i + rh) * 132 + 4 * c4]) = packed;
  }
  if (TRANSPOSED_COPY) {
    __syncthreads();
    // thread -> (tile column tc, 16-row chunk ch): gathers a column run and writes 16 bytes of qT
    for (int e = threadIdx.x; e < 128 * 8; e += 256) {
      const int tc = e >> 3, ch = e & 7;
      const int gc = c0 + tc, gr = wg.y * 128 + 16 * ch;
      if (gc < cols && gr < rows) {  // rows % 32 == 0: a 16-row chunk is entirely in or out
        uint32_t w[4];
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          uint32_t acc = 0;
#pragma unroll
          for (int b = 0; b < 4; ++b) acc |= (uint32_t)s_codes[(16 * ch + 4 * d + b) * 132 + tc] << (8 * b);
          w[d] = acc;
        }
        *reinterpret_cast<uint4*>(qT + (int64_t)gc * ldqT + gr) = make_uint4(w[0], w[1], w[2], w[3]);
      }
    }
  }
}

template <typename T, int B>
static void launch_quantize(const T* x, int64_t ldx, int rows, int cols, int8_t* q, int64_t ldq, float* s, int8_t* qT,
                            int64_t ldqT, float* sT, hipStream_t st) {
  dim3 grid(tile_grid((cols + 127) / 128, (rows + 127) / 128));
  if constexpr (B == 32) {
    if (!qT && grid.x < 512) {  // fewer than two workgroups per compute unit: one wave per workgroup instead
      hipLaunchKernelGGL((quantize_kernel<T, B, false, 1>), dim3(tile_grid((cols + 127) / 128, rows / 32)), dim3(64), 0, st, x,
                         ldx, rows, cols, q, ldq, s, qT, ldqT, sT);
      return;
    }
  }
  if (qT)
    hipLaunchKernelGGL((quantize_kernel<T, B, true>), grid, dim3(256), 0, st, x, ldx, rows, cols, q, ldq, s, qT, ldqT, sT);
  else
    hipLaunchKernelGGL((quantize_kernel<T, B, false>), grid, dim3(256), 0, st, x, ldx, rows, cols, q, ldq, s, qT, ldqT, sT);
}

template <typename T>
static void dispatch_quantize(int block, const T* x, int64_t ldx, int rows, int cols, int8_t* q, int64_t ldq, float* s,
                              int8_t* qT, int64_t ldqT, float* sT, hipStream_t st) {
  if (block == 32) launch_quantize<T, 32>(x, ldx, rows, cols, q, ldq, s, qT, ldqT, sT, st);
  else if (block == 64) launch_quantize<T, 64>(x, ldx, rows, cols, q, ldq, s, qT, ldqT, sT, st);
  else launch_quantize<T, 128>(x, ldx, rows, cols, q, ldq, s, qT, ldqT, sT, st);
}

// Dequantizer Q^-1 of Eq. 1: out = code * scale as FP32 or FP16 (the hand-over to a floating-point operator
// such as the FP16 attention core of Sec. 7.1).  A thread converts 16 consecutive codes of one row.
template <typename T>
__global__ void __launch_bounds__(256) dequantize_kernel(const int8_t* __restrict__ q, const float* __restrict__ s, int rows,
                                                          int cols, int block, T* __restrict__ out, int64_t ldo) {
  const int chunks = cols / 16;
  const int64_t total = (int64_t)rows * chunks;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int row = (int)(i / chunks), col = 16 * (int)(i % chunks);
    const uint4 p = *reinterpret_cast<const uint4*>(q + (int64_t)row * cols + col);
    const float sc = s[(int64_t)(row / block) * (cols / block) + col / block];
    const uint32_t w[4] = {p.x, p.y, p.z, p.w};
    float v[16];
#pragma unroll
    for (int d = 0; d < 4; ++d)
#pragma unroll
      for (int b = 0; b < 4; ++b) v[4 * d + b] = (float)(int8_t)(w[d] >> (8 * b)) * sc;
    T* dst = out + (int64_t)row * ldo + col;
    if constexpr (sizeof(T) == 4) {
#pragma unroll
      for (int d = 0; d < 4; ++d)
        *reinterpret_cast<float4*>(dst + 4 * d) = make_float4(v[4 * d], v[4 * d + 1], v[4 * d + 2], v[4 * d + 3]);
    } else {
      typedef _Float16 h8 __attribute__((ext_vector_type(8)));
#pragma unroll
      for (int d = 0; d < 2; ++d) {
        h8 h;
#pragma unroll
        for (int b = 0; b < 8; ++b) h[b] = (_Float16)v[8 * d + b];
        *reinterpret_cast<h8*>(dst + 8 * d) = h;
      }
    }
  }
}

}  // namespace jf

extern "C" int32_t jf_dequantize_block(const int8_t* q, const float* s, int64_t rows, int64_t cols, int32_t block,
                                       void* out, int32_t out_dtype, int64_t ldo, void* stream) {
  using namespace jf;
  if (!q || !s || !out) return JF_ERR_NULL;
  if (out_dtype != 0 && out_dtype != 1) return JF_ERR_DTYPE;
  if (!valid_block(block)) return JF_ERR_BLOCK;
  if (!valid_dim(rows, block) || !valid_dim(cols, block) || !valid_size(rows, cols) || ldo < cols) return JF_ERR_SHAPE;
  if (!aligned16(q) || !aligned4(s) || !aligned16(out) || (ldo % 8)) return JF_ERR_ALIGN;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const int64_t total = rows * (cols / 16);
  const unsigned grid = (unsigned)((total + 255) / 256 < 8192 ? (total + 255) / 256 : 8192);
  if (out_dtype == 0)
    hipLaunchKernelGGL((dequantize_kernel<float>), dim3(grid), dim3(256), 0, st, q, s, (int)rows, (int)cols, (int)block,
                       static_cast<float*>(out), ldo);
  else
    hipLaunchKernelGGL((dequantize_kernel<_Float16>), dim3(grid), dim3(256), 0, st, q, s, (int)rows, (int)cols, (int)block,
                       static_cast<_Float16*>(out), ldo);
  return launch_status();
}

extern "C" int32_t jf_quantize_block(const void* x, int32_t x_dtype, int64_t rows, int64_t cols, int64_t ldx,
                                     int32_t block, int8_t* q, int64_t ldq, float* s, int8_t* qT, int64_t ldqT,
                                     float* sT, void* stream) {
  using namespace jf;
  if (!x || !q || !s) return JF_ERR_NULL;
  if ((qT == nullptr) != (sT == nullptr)) return JF_ERR_NULL;
  if (x_dtype != 0 && x_dtype != 1) return JF_ERR_DTYPE;
  if (!valid_block(block)) return JF_ERR_BLOCK;
  if (!valid_dim(rows, block) || !valid_dim(cols, block) || !valid_size(rows, cols)) return JF_ERR_SHAPE;
  if (ldx < cols || ldq < cols || (qT && ldqT < rows)) return JF_ERR_SHAPE;
  if (!aligned16(x) || !aligned16(q) || !aligned4(s) || (ldx % 16) || (ldq % 16)) return JF_ERR_ALIGN;
  if (qT && (!aligned16(qT) || !aligned4(sT) || (ldqT % 16))) return JF_ERR_ALIGN;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (x_dtype == 0)
    dispatch_quantize<float>(block, static_cast<const float*>(x), ldx, (int)rows, (int)cols, q, ldq, s, qT, ldqT, sT, st);
  else
    dispatch_quantize<_Float16>(block, static_cast<const _Float16*>(x), ldx, (int)rows, (int)cols, q, ldq, s, qT, ldqT, sT, st);
  return launch_status();
}
