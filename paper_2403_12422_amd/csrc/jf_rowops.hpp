// Helpers shared by the INT8-in / INT8-out operators (Sec. 6, Alg. 2, App. A): unpacking and Eq. 1 for 16 codes at a
// time, the lane mapping of the block-32 strip kernels, and host-side argument checks.
#pragma once
#include "jf_common.hpp"

namespace jf {

__device__ __forceinline__ float amax4(float m, float a, float b, float c, float d) {
  return fmaxf(fmaxf(m, fmaxf(fabsf(a), fabsf(b))), fmaxf(fabsf(c), fabsf(d)));
}

__device__ __forceinline__ uint4 quantize16(const float (&y)[16], double inv) {
  uint4 o;
  o.x = quantize4(y[0], y[1], y[2], y[3], inv);
  o.y = quantize4(y[4], y[5], y[6], y[7], inv);
  o.z = quantize4(y[8], y[9], y[10], y[11], inv);
  o.w = quantize4(y[12], y[13], y[14], y[15], inv);
  return o;
}

// 16 codes -> (code + 128) as float: one XOR per dword flips the sign bits, then each byte converts
// with v_cvt_f32_ubyteN.  The caller folds the -128 into its fused multiply-add.
__device__ __forceinline__ void unpack16_biased(const uint4& p, float (&u)[16]) {
  const uint32_t w[4] = {p.x ^ 0x80808080u, p.y ^ 0x80808080u, p.z ^ 0x80808080u, p.w ^ 0x80808080u};
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    u[4 * d + 0] = (float)(w[d] & 0xffu);
    u[4 * d + 1] = (float)((w[d] >> 8) & 0xffu);
    u[4 * d + 2] = (float)((w[d] >> 16) & 0xffu);
    u[4 * d + 3] = (float)(w[d] >> 24);
  }
}

// Reduce over the lanes of a wave that share a quantization-block column in the (8 rows x 8 chunks)
// strip mapping: all 8 row lanes (bits 3..5) and the B/16 (<= 8) chunk lanes of the block (low bits).
template <int B>
__device__ __forceinline__ float strip_block_max(float m) {
  constexpr int CH = B >= 128 ? 7 : (B == 64 ? 3 : 1);
  return wave_group_max<56 | CH>(m);
}

// ------------------------------------------------------------------------------------------------
// Block size 32: the element-wise operators as one WAVE per workgroup.  A wave owns a strip of 32 rows x 128
// columns -- four quantization blocks side by side.  Lane l = (rsub = l / 8, ch = l % 8) holds the 16-byte chunk ch
// of rows rsub, rsub + 8, rsub + 16, rsub + 24 of the strip: every load or store instruction of the wave moves
// eight full 128-byte lines, a lane holds 64 elements of ONE block (columns 32 (ch / 2) .. + 31), so the block's
// max-abs is a local maximum followed by four cross-lane steps, and nothing is exchanged between waves: no LDS
// traffic (but the GELU tables), no barrier.  Per element the kernels spend what Alg. 2 needs (unpack, the
// operator, max-abs, Eq. 1) and little else; the per-lane overhead is paid once per 64 elements.
// Strips (waves) per workgroup: four neighbouring strips of the same rows, so that 512 contiguous bytes of every row
// are requested close together in time (on 0.8 GB tensors of 3072 columns 5.4-5.7 TB/s instead of 4.4-5.0 with one
// strip per workgroup).  The waves of a workgroup share nothing and never meet at a barrier.
constexpr int kStripWaves = 4;
struct Strip32 {
  int ch, rsub;     // chunk column and row of the lane inside an 8-row pass
  int bi, lc;       // block row of the strip, block columns of the matrix
  int c0, col;      // first column of the strip, first column of the lane's chunks
  bool ok;          // the lane's chunks lie inside the matrix (cols % 32 == 0: a block is all in or all out)
  int64_t base;     // element offset of the lane's chunk in pass 0; pass p adds 8 p cols.  Lanes outside the matrix
                    // point at the strip's first chunk instead: they load like the others (no branch), share their
                    // reductions only with each other (whole blocks are in or out), and store nothing.
  int lane, wave;   // lane of the wave, wave of the workgroup (a workgroup holds kStripWaves neighbouring strips)
  bool inside;      // the wave's strip exists (the last workgroup may hold fewer)
  __device__ __forceinline__ Strip32(int rows, int cols) {
    lane = threadIdx.x & 63;
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    ch = lane & 7;
    rsub = lane >> 3;
    const unsigned groups = (unsigned)((cols + 127) / 128), strips = groups * (unsigned)(rows / 32);
    const unsigned id = blockIdx.x * (blockDim.x >> 6) + wave;   // strips are numbered column group fastest
    inside = id < strips;
    const unsigned sid = inside ? id : strips - 1;
    c0 = (int)(sid % groups) * 128;
    bi = (int)(sid / groups);
    lc = cols / 32;
    col = c0 + 16 * ch;
    ok = col < cols;
    base = (int64_t)(bi * 32 + rsub) * cols + (ok ? col : c0);
  }
  // index of the lane's block in a scale grid (clamped like base)
  __device__ __forceinline__ int64_t block_index() const { return (int64_t)bi * lc + (ok ? col : c0) / 32; }
};

// max-abs of 16 values folded into m: eight v_max3_f32 with absolute-value modifiers (the compiler's fmaxf
// quiets each operand with an extra instruction first)
__device__ __forceinline__ float amax16(float m, const float (&y)[16]) {
#pragma unroll
  for (int e = 0; e < 16; e += 2) asm("v_max3_f32 %0, |%1|, |%2|, %0" : "+v"(m) : "v"(y[e]), "v"(y[e + 1]));
  return m;
}

// Block max-abs over the 16 lanes of a strip that share a block column (same ch / 2), then Eq. 1's scale.
__device__ __forceinline__ void strip32_block_scale(float m, float& scale, double& inv) {
  m = wave_group_max<56 | 1>(m);
  block_scale(m, scale, inv);
}

__device__ __forceinline__ void load16f(const float* p, float (&v)[16]) {
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const float4 t = *reinterpret_cast<const float4*>(p + 4 * d);
    v[4 * d] = t.x; v[4 * d + 1] = t.y; v[4 * d + 2] = t.z; v[4 * d + 3] = t.w;
  }
}

// ------------------------------------------------------------------------------------------------ host
// workgroups of the strip kernels: kStripWaves strips each
static inline dim3 strip_grid(int64_t rows, int64_t cols) {
  const int64_t strips = ((cols + 127) / 128) * (rows / 32);
  return dim3((unsigned)((strips + kStripWaves - 1) / kStripWaves));
}

static inline int32_t check_eltwise(const void* x, const void* sx, const void* y, const void* sy, int64_t N, int64_t C,
                             int32_t block) {
  if (!x || !sx || !y || !sy) return JF_ERR_NULL;
  if (!valid_block(block)) return JF_ERR_BLOCK;
  if (!valid_dim(N, block) || !valid_dim(C, block) || !valid_size(N, C)) return JF_ERR_SHAPE;
  if (!aligned16(x) || !aligned4(sx) || !aligned16(y) || !aligned4(sy)) return JF_ERR_ALIGN;
  return JF_OK;
}

}  // namespace jf
