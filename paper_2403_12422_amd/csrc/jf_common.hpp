// Shared device / host helpers of the gfx950 per-block INT8 library.
// Wavefront = 64 lanes everywhere in this file.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "jetfire.h"

namespace jf {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------- host side
extern thread_local int32_t g_last_hip_error;

inline int32_t launch_status() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    g_last_hip_error = (int32_t)e;
    return JF_ERR_LAUNCH;
  }
  return JF_OK;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool aligned4(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }
inline bool valid_block(int32_t b) { return b == 32 || b == 64 || b == 128; }
// Dimensions are kept below 2^24 so that every index fits an int32 after
// division by the block size and element offsets fit 48 bits.
// Rows of dgamma | dbeta partial sums that the LayerNorm backward kernels leave in the workspace.  Up to 2048
// columns a workgroup walks over the row blocks it owns and leaves one row (at most two workgroups per compute
// unit); wider rows use one workgroup per row block, which leaves four.
inline int64_t ln_bwd_partial_rows(int64_t N, int64_t C, int32_t block) {
  if (C > 2048) return (N / block) * 4;
  return N / block < 512 ? N / block : 512;
}
inline bool valid_dim(int64_t d, int32_t block) { return d > 0 && d <= (int64_t(1) << 24) && d % block == 0; }

// -------------------------------------------------------------- device side
// Max over the lanes whose ids differ only in the bits of `mask` (butterfly
// over ds_bpermute; every lane of the wave must be active).
template <int MASK>
__device__ __forceinline__ float wave_group_max(float v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1)
    if (MASK & m) v = fmaxf(v, __shfl_xor(v, m, 64));
  return v;
}

template <int MASK>
__device__ __forceinline__ float wave_group_sum(float v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1)
    if (MASK & m) v += __shfl_xor(v, m, 64);
  return v;
}

template <int MASK>
__device__ __forceinline__ double wave_group_sum_f64(double v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1)
    if (MASK & m) v += __shfl_xor(v, m, 64);
  return v;
}

// Eq. 1 scale of a block from its max-abs: one IEEE FP32 division; 0 for an
// all-zero block.  `inv` is the factor codes are multiplied with (0 if the
// block is all zero, so that every code becomes 0).
__device__ __forceinline__ void block_scale(float amax, float& scale, float& inv) {
  scale = amax / 127.0f;
  inv = amax > 0.0f ? 1.0f / scale : 0.0f;
}

// round-half-even(x * inv) as an integer in the low byte of the result:
// adding 1.5 * 2^23 inside one fused multiply-add leaves the rounded integer
// in the low mantissa bits (two's complement modulo 256 in bits 0..7).
__device__ __forceinline__ uint32_t code_bits(float x, float inv) {
  return __float_as_uint(__builtin_fmaf(x, inv, 12582912.0f));
}

// Pack the low bytes of four code_bits() results into one dword, a0 lowest.
__device__ __forceinline__ uint32_t pack_codes(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3) {
  uint32_t lo = __builtin_amdgcn_perm(a1, a0, 0x0c0c0400u);  // [a0.b0, a1.b0, 0, 0]
  uint32_t hi = __builtin_amdgcn_perm(a3, a2, 0x04000c0cu);  // [0, 0, a2.b0, a3.b0]
  return lo | hi;
}

__device__ __forceinline__ uint32_t quantize4(float x0, float x1, float x2, float x3, float inv) {
  return pack_codes(code_bits(x0, inv), code_bits(x1, inv), code_bits(x2, inv), code_bits(x3, inv));
}

// Signed byte k (0..3) of a packed dword as float.
__device__ __forceinline__ float byte_to_float(uint32_t packed, int k) {
  return (float)((int32_t)(packed << (24 - 8 * k)) >> 24);
}

}  // namespace jf
