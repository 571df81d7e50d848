// Shared device / host helpers of the gfx950 per-block INT8 library.
// Wavefront = 64 lanes everywhere in this file.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

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
// Rows of dgamma | dbeta partial sums that the first kernel of LayerNorm backward leaves in the workspace: one per
// workgroup, which walks over the groups of 32 rows it owns (at most 512 workgroups).
inline int64_t ln_bwd_partial_rows(int64_t N) { return N / 32 < 512 ? N / 32 : 512; }
// Workspace of LayerNorm backward: the partial rows (dgamma | dbeta, 2 C floats each), and behind them the two row means
// of every row that the first kernel hands to the second (one pair per range of 2048 columns).
inline size_t ln_bwd_workspace_bytes(int64_t N, int64_t C) {
  return (size_t)ln_bwd_partial_rows(N) * 2 * (size_t)C * sizeof(float) + (size_t)N * 2 * sizeof(float) * (size_t)((C + 2047) / 2048);
}
inline bool valid_dim(int64_t d, int32_t block) { return d > 0 && d <= (int64_t(1) << 24) && d % block == 0; }
// A tensor holds at most 2^40 elements (far beyond any device memory): keeps every workgroup count inside 32 bits.
inline bool valid_size(int64_t rows, int64_t cols) { return rows * cols <= (int64_t(1) << 40); }

// -------------------------------------------------------------- device side
// The kernels that tile a matrix in two dimensions are launched as a one-dimensional grid, column group fastest:
// the y and z dimensions of a grid stop at 65535, which a tensor of 2^24 rows exceeds.
struct TileIndex {
  int x, y;  // column group, row group
};
__device__ __forceinline__ TileIndex tile_of_workgroup(int column_groups) {
  const unsigned i = blockIdx.x;
  TileIndex t;
  t.x = (int)(i % (unsigned)column_groups);
  t.y = (int)(i / (unsigned)column_groups);
  return t;
}
// host side: workgroups of such a launch
inline unsigned tile_grid(int64_t column_groups, int64_t row_groups) { return (unsigned)(column_groups * row_groups); }

// Cross-lane exchange for butterfly reductions without LDS traffic: the value of lane (id ^ 2^BIT) for every lane.
// Bits 0..3 are DPP moves inside a row of 16 lanes (quad permutes, half-row mirror, row rotate by 8); bits 4 and 5
// use the row / half-wave swap instructions of gfx950.  BIT 2 (half-row mirror, lane i <-> 7 - i) equals
// "xor 4" only when the four lanes of every quad already hold the same value, i.e. after the steps for bits 0
// and 1 -- every reduction below that contains bit 2 also contains bits 0 and 1 and takes them first.
// Every lane of the wave must be active.
template <int BIT>
__device__ __forceinline__ int lane_xor_i32(int v) {
  if constexpr (BIT == 0) return __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false);        // quad_perm [1,0,3,2]
  else if constexpr (BIT == 1) return __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
  else if constexpr (BIT == 2) return __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, false);  // row_half_mirror
  else if constexpr (BIT == 3) return __builtin_amdgcn_update_dpp(0, v, 0x128, 0xf, 0xf, false);  // row_ror:8
  else if constexpr (BIT == 4) {
    // odd rows of the first operand <-> even rows of the second: (r0 r0 r2 r2) and (r1 r1 r3 r3)
    auto p = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return ((__lane_id() >> 4) & 1) ? (int)p[0] : (int)p[1];
  } else {
    // upper half of the first operand <-> lower half of the second: (lo lo) and (hi hi)
    auto p = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return (__lane_id() >> 5) ? (int)p[0] : (int)p[1];
  }
}
template <int BIT>
__device__ __forceinline__ float lane_xor_f32(float v) {
  return __builtin_bit_cast(float, lane_xor_i32<BIT>(__builtin_bit_cast(int, v)));
}
template <int BIT>
__device__ __forceinline__ double lane_xor_f64(double v) {
  const long long b = __builtin_bit_cast(long long, v);
  const unsigned lo = (unsigned)lane_xor_i32<BIT>((int)(b & 0xffffffffll)), hi = (unsigned)lane_xor_i32<BIT>((int)(b >> 32));
  return __builtin_bit_cast(double, ((long long)hi << 32) | (long long)lo);
}

template <int MASK, int BIT = 0, class T, class Op, class Xor>
__device__ __forceinline__ T wave_group_reduce(T v, Op op, Xor lane_xor) {
  static_assert(!(MASK & 4) || (MASK & 3) == 3, "the step for bit 2 needs bits 0 and 1 reduced first");
  if constexpr (BIT < 6) {
    if constexpr ((MASK >> BIT) & 1) v = op(v, lane_xor(v, std::integral_constant<int, BIT>()));
    return wave_group_reduce<MASK, BIT + 1>(v, op, lane_xor);
  } else {
    return v;
  }
}

// Max / sum over the lanes whose ids differ only in the bits of MASK (butterfly; every lane of the wave must be
// active).  The summation order is fixed, so results are bit-stable.
template <int MASK>
__device__ __forceinline__ float wave_group_max(float v) {
  return wave_group_reduce<MASK>(v, [](float a, float b) { return fmaxf(a, b); },
                                 [](float x, auto bit) { return lane_xor_f32<decltype(bit)::value>(x); });
}

template <int MASK>
__device__ __forceinline__ float wave_group_sum(float v) {
  return wave_group_reduce<MASK>(v, [](float a, float b) { return a + b; },
                                 [](float x, auto bit) { return lane_xor_f32<decltype(bit)::value>(x); });
}

template <int MASK>
__device__ __forceinline__ double wave_group_sum_f64(double v) {
  return wave_group_reduce<MASK>(v, [](double a, double b) { return a + b; },
                                 [](double x, auto bit) { return lane_xor_f64<decltype(bit)::value>(x); });
}

// Eq. 1 scale of a block from its max-abs: one IEEE FP32 division; 0 for an all-zero block.  `inv` is the
// reciprocal of the scale in double precision (0 for an all-zero block, so that every code becomes 0): the
// hardware estimate refined by two Newton steps, relative error below 2^-50.  The double reciprocal exists for
// every FP32 scale, subnormal ones included.
__device__ __forceinline__ void block_scale(float amax, float& scale, double& inv) {
  scale = amax / 127.0f;
  const double s = (double)scale;
  double r = __builtin_amdgcn_rcp(s);
  r = __builtin_fma(__builtin_fma(-s, r, 1.0), r, r);
  r = __builtin_fma(__builtin_fma(-s, r, 1.0), r, r);
  inv = scale > 0.0f ? r : 0.0;
}

// round-half-even(x / scale) of the EXACT quotient of the two FP32 numbers (Eq. 1), as an integer in the low
// byte of the result.  A quotient of two FP32 numbers is either exactly k + 1/2 or at least 2^-26 away from it,
// so it suffices to know it to better than that, which x * inv in double does (error below 127.5 * 2^-50):
//   t1 = fma(x, inv, 1.5 * 2^20)    lies in one binade with ulp 2^-32: everything within 2^-33 of k + 1/2 -- only
//                                   exact ties are -- lands exactly on the tie, everything else stays on its side;
//   t  = t1 + (1.5 * 2^52 - 1.5 * 2^20)   rounds to an integer, the exact tie to even (1.5 * 2^52 is even), and
//                                   leaves it in the low mantissa bits (two's complement modulo 256 in bits 0..7).
// An FP32 product x * (1/scale) cannot do this: its error of up to 7.6e-6 decides every tie and near-tie at
// random, and tensors whose blocks keep their scale through an operator consist of little else.
__device__ __forceinline__ uint32_t code_bits(float x, double inv) {
  const double t1 = __builtin_fma((double)x, inv, 1572864.0);
  const double t = t1 + (6755399441055744.0 - 1572864.0);
  return (uint32_t)__builtin_bit_cast(unsigned long long, t);
}

// Pack the low bytes of four code_bits() results into one dword, a0 lowest.
__device__ __forceinline__ uint32_t pack_codes(uint32_t a0, uint32_t a1, uint32_t a2, uint32_t a3) {
  uint32_t lo = __builtin_amdgcn_perm(a1, a0, 0x0c0c0400u);  // [a0.b0, a1.b0, 0, 0]
  uint32_t hi = __builtin_amdgcn_perm(a3, a2, 0x04000c0cu);  // [0, 0, a2.b0, a3.b0]
  return lo | hi;
}

__device__ __forceinline__ uint32_t quantize4(float x0, float x1, float x2, float x3, double inv) {
  return pack_codes(code_bits(x0, inv), code_bits(x1, inv), code_bits(x2, inv), code_bits(x3, inv));
}

// Signed byte k (0..3) of a packed dword as float.
__device__ __forceinline__ float byte_to_float(uint32_t packed, int k) {
  return (float)((int32_t)(packed << (24 - 8 * k)) >> 24);
}

}  // namespace jf
