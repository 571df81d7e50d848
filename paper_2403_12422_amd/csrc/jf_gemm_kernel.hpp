// Per-block INT8 linear layer (Sec. 5, Alg. 1): forward, dgrad, wgrad and the INT32-partial test hook.
//
// All three products are one kernel in the canonical form  out = A * Bm^T
// (A: M x K, Bm: Nn x K) with two storage modes per operand:
//   K-major  : rows indexed by the output dimension, contraction dimension contiguous
//              (X and W in the forward product, dY in dgrad);
//   M-major  : rows indexed by the contraction dimension (W in dgrad, dY and X in wgrad).
// Tiles are copied global -> LDS unchanged; an M-major tile is transposed
// byte-wise while it is read back with ds_read_b64_tr_b8, so the backward
// products need no separate transpose pass and no re-quantization (square
// blocks: the scale grid is simply indexed with swapped strides).
//
// Per 32-wide K step each wave issues one v_mfma_i32_32x32x32_i8 per 32x32
// output sub-block; at the end of every quantization block along K the INT32
// tile is folded into the FP32 accumulator as fma(sA*sB, (float)v, acc)
// (Sec. 5.3), and after the K loop the accumulator is quantized per block
// (Eq. 1) in registers.  The MFMA operands are swapped (rows of Bm feed the
// "A" port) so that a lane ends up with 4 consecutive output columns of one
// output row per register quad: codes pack into dwords without shuffles.
#pragma once
#include <algorithm>
#include <atomic>
#include <cmath>
#include <type_traits>

#include "jf_common.hpp"

namespace jf {

struct GemmArgs {
  const int8_t* A;
  const int8_t* Bm;
  const float* SA;
  const float* SB;
  int M, Nn, K;        // output M x Nn, contraction length K
  int64_t lda, ldb;    // leading dimensions (bytes) of the operands as stored
  int sa_p, sa_k;      // element strides of SA for (output block row, K block)
  int sb_p, sb_k;      // element strides of SB for (output block col, K block)
  int8_t* Oq;          // M x Nn codes (nullable)
  float* Os;           // (M/B) x (Nn/B) scales (nullable with Oq)
  float* Of;           // M x Nn FP32 accumulator (nullable)
  int32_t* dump;       // test hook: INT32 partials of K block dump_kb
  int dump_kb;
};

// ---------------------------------------------------------------------------------------------
// LDS staging.  A stage holds KC bytes of K for both operand tiles: KC = 64 (two MFMA K steps), or
// 128 for B = 128 so that a stage always holds whole quantization blocks and block boundaries are
// known at compile time.  Tiles go global -> LDS with global_load_lds_dwordx4: no VGPR staging, no
// ds_write; the 64 lanes of one such instruction fill 64 consecutive 16-byte LDS slots, so the
// layout cannot be padded.  Bank conflicts are avoided by an XOR swizzle instead: the tile is a
// matrix of 16-byte chunks with CPR chunks per row, and chunk c of row r lives in slot
// r*CPR + (c ^ swz(r)); swz is chosen per operand layout so that the lanes one fragment read serves per
// clock (16 rows for ds_read_b128 of a K-major operand, 8 rows for ds_read_b64_tr_b8 of an M-major one)
// fall into different bank groups.
template <int TILE, bool KMAJOR, int KC>
struct TileLayout {
  static constexpr int kRows = KMAJOR ? TILE : KC;            // LDS rows: output rows, or K rows
  static constexpr int kCPR = (KMAJOR ? KC : TILE) / 16;      // 16-byte chunks per LDS row
  static constexpr int kSlots = kRows * kCPR;
  static_assert(kCPR == 4 || kCPR == 8 || kCPR == 16, "rows of 64, 128 or 256 bytes");
  // K-major tiles are read with ds_read_b128, which serves 16 lanes (16 consecutive rows, one chunk each) per
  // clock from 256 bytes of banks: the 16 rows must land in 16 different 16-byte bank groups.  A row of 128
  // (64) bytes starts at bank group 8*(r%2) (4*(r%4)), so the XOR term has to run through its 8 (4) values
  // over the rows that share that start.  M-major tiles are read with 8-byte transposing reads, 8 rows per
  // 16 lanes: 8 consecutive rows at a fixed chunk cover 8 bank groups.
  static __device__ __forceinline__ int swz(int r) {
    if (KMAJOR) return (r / (16 / kCPR)) % kCPR;
    return (r / (kCPR == 4 ? 2 : 1)) % (kCPR == 16 ? 8 : kCPR);
  }
  static __device__ __forceinline__ int slot(int r, int c) { return r * kCPR + (c ^ swz(r)); }
  // LDS bytes when the tile is filled by whole 64-lane load instructions of NW waves (the tail is padding)
  static constexpr int bytes(int nw) { return ((kSlots + 64 * nw - 1) / (64 * nw)) * (64 * nw) * 16; }
};

typedef __attribute__((address_space(3))) void* lds_ptr;
typedef const __attribute__((address_space(1))) void* gbl_ptr;
typedef __attribute__((address_space(3))) v2i* lds_v2i;
typedef __attribute__((address_space(3))) v4i* lds_v4i;
typedef float v4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) v4f* lds_v4f;

// Per-lane LDS byte offsets of an operand's MFMA fragments inside a stage buffer.  Everything that
// does not depend on the lane is a compile-time immediate added at the read, so the main loop spends
// no vector ALU on addressing.  K-major: the K step j toggles a swizzled chunk bit (one offset per
// j) and the sub-tile adds a constant; M-major: the sub-tile toggles swizzled bits (one offset per
// sub-tile of the wave) and the K step adds a constant.
template <int TILE, bool KMAJOR, int KC, int NSUB>
struct FragAddr {
  typedef TileLayout<TILE, KMAJOR, KC> L;
  static constexpr int kN = KMAJOR ? KC / 32 : NSUB;
  int off[kN];
  __device__ __forceinline__ void init(int sub0, int lane) {
    if (KMAJOR) {
#pragma unroll
      for (int j = 0; j < kN; ++j) off[j] = 16 * L::slot(sub0 * 32 + (lane & 31), 2 * j + (lane >> 5));
    } else {
      // ds_read_b64_tr_b8: within 16 lanes, lane 2r+h points at 8 bytes (columns 8h..8h+7) of row r;
      // lane c receives column c of that 8 x 16 byte matrix.  Two reads give 16 consecutive K.
      const int i = lane & 15, g = lane >> 4;
#pragma unroll
      for (int u = 0; u < kN; ++u)
        off[u] = 16 * L::slot(16 * (g >> 1) + (i >> 1), (sub0 + u) * 2 + (g & 1)) + 8 * (i & 1);
    }
  }
  // fragment of sub-tile u (relative to the wave's first), K step j, from the stage buffer at `tile`
  __device__ __forceinline__ v4i read(const int8_t* tile, int u, int j) const {
    if (KMAJOR) {
      return *(lds_v4i)(tile + off[j] + u * (32 * L::kCPR * 16));
    } else {
      const int8_t* p = tile + off[u] + j * (32 * L::kCPR * 16);
      v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i)(p));
      v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i)(p + 8 * L::kCPR * 16));
      v4i r = {lo[0], lo[1], hi[0], hi[1]};
      return r;
    }
  }
};

// One direct-to-LDS load of 16 bytes per lane: lane l's bytes from ubase + voff go to LDS address lds + 16*l.
// Written out because the compiler only selects the 64-bit per-lane address form for the builtin; the form with
// a scalar base and a 32-bit vector offset needs no address arithmetic on the vector ALU.  M0 carries the LDS
// address and needs one wait state before the load reads it.  The load counts in vmcnt like any other; the
// callers wait for it with s_waitcnt before the stage barrier.
// Every direct-to-LDS load of the kernel goes through these two helpers, so the compiler itself never uses M0.
__device__ __forceinline__ uint32_t lds_address(const int8_t* lds_tile, int lds_byte) {
  // the tile's LDS address is taken before the byte offset is added: a cast of the sum would carry a null check
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_ptr)(lds_tile) + (uint32_t)lds_byte);
}
__device__ __forceinline__ void load_lds_16(const int8_t* ubase, uint32_t voff, const int8_t* lds_tile, int lds_byte) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(voff), "s"(ubase), "s"(lds_address(lds_tile, lds_byte))
               : "memory", "m0");
}
// the same with a full 64-bit address per lane (the clamped last stage of a K that is not a multiple of the stage)
__device__ __forceinline__ void load_lds_16_vaddr(const int8_t* vaddr, const int8_t* lds_tile, int lds_byte) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :
               : "v"(vaddr), "s"(lds_address(lds_tile, lds_byte))
               : "memory", "m0");
}
// A pointer that is the same for all lanes, moved to scalar registers for good.
__device__ __forceinline__ const int8_t* uniform_pointer(const int8_t* p) {
  const uint64_t v = (uint64_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return (const int8_t*)(((uint64_t)hi << 32) | lo);
}

// Global byte offset of the chunk that belongs in LDS slot `slot_idx` of a stage starting at K offset k0.
// Out-of-range rows / columns / K are clamped to valid addresses: what they deliver only reaches
// outputs that are never stored (or K steps that are never run), so no zero fill is needed.
template <int TILE, bool KMAJOR, int KC>
__device__ __forceinline__ int64_t chunk_offset(int slot_idx, int o0, int k0, int outer_dim, int K, int64_t ld) {
  typedef TileLayout<TILE, KMAJOR, KC> L;
  const int r = min(slot_idx / L::kCPR, L::kRows - 1);  // slots past the tile are padding: any valid source will do
  const int c = (slot_idx % L::kCPR) ^ L::swz(r);
  if (KMAJOR) {
    const int row = min(o0 + r, outer_dim - 1), kk = min(k0 + 16 * c, K - 16);
    return (int64_t)row * ld + kk;
  } else {
    const int krow = min(k0 + r, K - 1), col = min(o0 + 16 * c, outer_dim - 16);
    return (int64_t)krow * ld + col;
  }
}

// f(integral_constant<int, I>) for I = BEGIN .. END-1, unrolled at compile time
template <int BEGIN, int END, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (BEGIN < END) {
    f(std::integral_constant<int, BEGIN>());
    static_for<BEGIN + 1, END>(f);
  }
}

// acc += t * (float)v for one 32x32 sub-block (Sec. 5.3): 16 int->float conversions and 16 FMAs per lane.
// The fused multiply-add is written as v_fmac_f32 so that it updates the accumulator register in place;
// left to itself the register allocator ping-pongs the 64 accumulators between two register sets.
template <int R0 = 0, int R1 = 16>
__device__ __forceinline__ void fold(float (&acc)[16], const v16i& v, float t) {
#pragma unroll
  for (int r = R0; r < R1; ++r) {
    const float c = (float)v[r];
    asm("v_fmac_f32 %0, %1, %2" : "+v"(acc[r]) : "v"(t), "v"(c));
  }
}

// Compile-time shape of one kernel instance: tile, stage and LDS ring.
// DEEP: a stage of 128 K bytes where the shape's default is 64.
template <int B, int WM, int WN, int WGM, int WGN, bool AK, bool BK, bool DEEP>
struct GemmShape {
  static constexpr int NW = WGM * WGN;
  static constexpr int TM = 32 * WM * WGM, TN = 32 * WN * WGN;
  // K bytes per stage: 128 when a stage has to hold a whole B = 128 block, for the workgroups of more than
  // four waves of fewer than four sub-blocks each (one workgroup per compute unit, whose barriers are the most
  // expensive), and for the one-sub-block waves at B = 64 (a stage must hold an even number of sub-block x
  // K-block units); 64 otherwise, which lets three workgroups with a ring of three stages share the LDS of a
  // compute unit.
  static constexpr int KC = (DEEP || B == 128 || (WGM * WGN > 4 && WM * WN < 4) || (B == 64 && WM * WN == 1)) ? 128 : 64;
  typedef TileLayout<TM, AK, KC> LA;
  typedef TileLayout<TN, BK, KC> LB;
  static constexpr int A_BYTES = LA::bytes(NW), B_BYTES = LB::bytes(NW);
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  // Stages in the LDS ring: one being read, the rest in flight.  Tiles that leave a compute unit to a single
  // workgroup (more than four waves) take a ring of four if that fits the LDS, the others a ring of three.
  static constexpr int NBUF = (NW > 4 && 4 * STAGE_BYTES <= 156 * 1024) ? 4 : 3;
  static_assert(NBUF * STAGE_BYTES <= 160 * 1024, "the ring must fit the LDS of a compute unit");
  static constexpr int RING_BYTES = NBUF * STAGE_BYTES;
};

// One output tile: K loop and epilogue.  `tile_index` of `ntiles` is this workgroup's position in the launch (or in
// its part of a launch that holds two products); s_ring is the workgroup's LDS ring of NBUF stages, s_amax its
// max-abs exchange area, both owned by the calling kernel.
template <int B, int WM, int WN, int WGM, int WGN, bool AK, bool BK, bool DUMP, bool DEEP>
__device__ __forceinline__ void gemm_tile(const GemmArgs& g, const int tile_index, const int ntiles, int8_t* const s_ring,
                                          float (*const s_amax)[8]) {
  typedef GemmShape<B, WM, WN, WGM, WGN, AK, BK, DEEP> Shape;
  constexpr int NW = Shape::NW;
  constexpr int TM = Shape::TM, TN = Shape::TN;
  constexpr int KPB = B / 32;  // MFMA K steps per quantization block
  constexpr int KC = Shape::KC;
  constexpr int SPS = KC / 32;  // MFMA K steps per stage
  constexpr int NTILE = WM * WN;
  typedef typename Shape::LA LA;
  typedef typename Shape::LB LB;
  constexpr int A_BYTES = Shape::A_BYTES, B_BYTES = Shape::B_BYTES;
  constexpr int CA = A_BYTES / (1024 * NW), CB = B_BYTES / (1024 * NW);  // load instructions per wave and stage
  static_assert(B == 32 || (TM % B == 0 && TN % B == 0), "tile must hold whole quantization blocks");
  constexpr int STAGE_BYTES = Shape::STAGE_BYTES;
  constexpr int NBUF = Shape::NBUF;
  static_assert(TM / 32 <= 8 && TN / 32 <= 8, "max-abs exchange area");
  int8_t* const s_tile0 = s_ring;
  int8_t* const s_tile1 = s_ring + STAGE_BYTES;
  int8_t* const s_tile2 = s_ring + 2 * STAGE_BYTES;
  int8_t* const s_tile3 = s_ring + (NBUF > 3 ? 3 : 2) * STAGE_BYTES;
  auto tile_buf = [&](int buf) -> int8_t* {
    return buf == 0 ? s_tile0 : (buf == 1 ? s_tile1 : (buf == 2 ? s_tile2 : s_tile3));
  };

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;  // first 32-granule of this wave inside the tile

  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Renumber them so that every XCD
  // works on one contiguous run of tiles, and order the tiles in groups of GROUP_M tile rows, column by column
  // inside a group: the workgroups that are resident on an XCD at the same time then form a compact patch
  // (8 tile rows x a few tile columns) that re-reads few distinct operand tiles from that XCD's L2.
  constexpr int GROUP_M = TM >= 256 ? 4 : 8;
  const int tiles_n = (g.Nn + TN - 1) / TN, tiles_m = (g.M + TM - 1) / TM;
  const int xcd = tile_index & 7, idx = tile_index >> 3;
  const int tile = xcd * (ntiles >> 3) + min(xcd, ntiles & 7) + idx;
  const int group = tile / (GROUP_M * tiles_n), first_m = group * GROUP_M;
  const int in_group = tile - group * GROUP_M * tiles_n, group_rows = min(GROUP_M, tiles_m - first_m);
  const int m0 = (first_m + in_group % group_rows) * TM, n0 = (in_group / group_rows) * TN;

  const int nsteps = g.K / 32;
  const int nstages = (g.K + KC - 1) / KC;

  // A load's address is a workgroup-uniform base (the tile's origin, advanced by k0 (K-major) or k0*ld (M-major)
  // per stage with scalar instructions) plus a loop-invariant per-lane byte offset.  The offset fits 32 bits: a
  // tile spans at most 256 rows (or 128 K rows) of at most 2^24 + 32 bytes.  The load takes them as scalar base
  // + vector offset, so the K loop spends no vector ALU on addresses.
  uint32_t offA[CA], offB[CB];
  const int64_t originA = AK ? (int64_t)m0 * g.lda : (int64_t)m0, originB = BK ? (int64_t)n0 * g.ldb : (int64_t)n0;
#pragma unroll
  for (int i = 0; i < CA; ++i)
    offA[i] = (uint32_t)(chunk_offset<TM, AK, KC>((i * NW + wave) * 64 + lane, m0, 0, g.M, g.K, g.lda) - originA);
#pragma unroll
  for (int i = 0; i < CB; ++i)
    offB[i] = (uint32_t)(chunk_offset<TN, BK, KC>((i * NW + wave) * 64 + lane, n0, 0, g.Nn, g.K, g.ldb) - originB);
  const int8_t* const baseA = uniform_pointer(g.A + originA);
  const int8_t* const baseB = uniform_pointer(g.Bm + originB);
  const int64_t kstrideA = AK ? 1 : g.lda, kstrideB = BK ? 1 : g.ldb;
  // Block scales are wave-uniform: they are read with scalar loads straight into SGPRs, ahead of their use,
  // so they cost neither LDS traffic nor vector-memory slots.  Index [a][j]: sub-tile a of the wave,
  // quantization block j of the stage along K.  Granules outside the matrix are clamped (their products are unused).
  float sa_c[WM][SPS / KPB], sb_c[WN][SPS / KPB], sa_n[WM][SPS / KPB], sb_n[WN][SPS / KPB];
  int sa_row[WM], sb_row[WN];
#pragma unroll
  for (int a = 0; a < WM; ++a) sa_row[a] = (min(m0 + 32 * (wm0 + a), g.M - 32) / B) * g.sa_p;
#pragma unroll
  for (int b = 0; b < WN; ++b) sb_row[b] = (min(n0 + 32 * (wn0 + b), g.Nn - 32) / B) * g.sb_p;
  // The grids are read through the constant address space: they are never written by this kernel, and a
  // uniform load from that space is selected as a scalar load.
  typedef const __attribute__((address_space(4))) float* const_f32_ptr;
  const const_f32_ptr SAc = (const_f32_ptr)g.SA, SBc = (const_f32_ptr)g.SB;
  auto rotate_scales = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < SPS / KPB; ++j) {
#pragma unroll
      for (int a = 0; a < WM; ++a) sa_c[a][j] = sa_n[a][j];
#pragma unroll
      for (int b = 0; b < WN; ++b) sb_c[b][j] = sb_n[b][j];
    }
  };

  // Issue the direct-to-LDS loads of the stage that starts at K offset k0 into ring slot buf.
  // known_whole: the caller guarantees k0 + KC <= K (keeps the clamping path out of the loops).
  auto issue_at = [&](int k0, int buf, auto known_whole) __attribute__((always_inline)) {
    int8_t* ta = tile_buf(buf);
    if (known_whole || k0 + KC <= g.K) {
      const int8_t* const sa = baseA + k0 * kstrideA;
      const int8_t* const sb = baseB + k0 * kstrideB;
#pragma unroll
      for (int i = 0; i < CA; ++i) load_lds_16(sa, offA[i], ta, 1024 * (i * NW + wave));
#pragma unroll
      for (int i = 0; i < CB; ++i) load_lds_16(sb, offB[i], ta, A_BYTES + 1024 * (i * NW + wave));
    } else {  // the last stage of a K that is not a multiple of KC: clamp what lies beyond K
#pragma unroll
      for (int i = 0; i < CA; ++i) {
        const int64_t off = chunk_offset<TM, AK, KC>((i * NW + wave) * 64 + lane, m0, k0, g.M, g.K, g.lda);
        load_lds_16_vaddr(g.A + off, ta, 1024 * (i * NW + wave));
      }
#pragma unroll
      for (int i = 0; i < CB; ++i) {
        const int64_t off = chunk_offset<TN, BK, KC>((i * NW + wave) * 64 + lane, n0, k0, g.Nn, g.K, g.ldb);
        load_lds_16_vaddr(g.Bm + off, ta, A_BYTES + 1024 * (i * NW + wave));
      }
    }
  };

  FragAddr<TM, AK, KC, WM> addrA;
  FragAddr<TN, BK, KC, WN> addrB;
  addrA.init(wm0, lane);
  addrB.init(wn0, lane);

  float acc[WM][WN][16];
#pragma unroll
  for (int a = 0; a < WM; ++a)
#pragma unroll
    for (int b = 0; b < WN; ++b)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;
  const v16i zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};

  auto dump_tile = [&](const v16i& v, int a, int b) __attribute__((always_inline)) {
    const int m = m0 + 32 * (wm0 + a) + (lane & 31);
    const int nb = n0 + 32 * (wn0 + b) + 4 * (lane >> 5);
    if (m < g.M && nb < g.Nn) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        v4i o = {v[4 * q4], v[4 * q4 + 1], v[4 * q4 + 2], v[4 * q4 + 3]};
        *reinterpret_cast<v4i*>(g.dump + (int64_t)m * g.Nn + nb + 8 * q4) = o;
      }
    }
  };

  // Stage loop over the ring of NBUF LDS buffers: while stage s is computed, stages s+1 .. s+NBUF-1
  // are in flight, which covers the L2 latency even when a stage is only two K steps long.  The loop
  // is unrolled NBUF times so that every LDS address is a compile-time immediate and the accumulators
  // stay in the same registers; the last (at most NBUF) stages run from a generic copy after the loop.
  constexpr int LOADS = CA + CB;   // vector-memory instructions per wave and stage
  constexpr int AHEAD = NBUF - 1;  // stages issued ahead of the one being computed
  static_assert(LOADS * (AHEAD - 1) <= 63, "vmcnt immediate");
  // End of a stage: wait for this wave's own loads of the stage that is read next, then meet the other waves.
  // A bare s_barrier is used instead of __syncthreads(): the fence of the latter makes the compiler drain
  // every outstanding load (vmcnt(0)), including the stage that is meant to stay in flight.  Ordering is kept
  // by hand: the asm is a compiler barrier for memory accesses, each wave has consumed all its LDS reads of the
  // finished stage before it arrives, and direct-to-LDS loads are counted by vmcnt.  The wait itself is the
  // s_waitcnt builtin, which the compiler's own counter tracking understands: it then knows that the loads of
  // the stage read next have landed and adds no drain of its own in front of the fragment reads.
  // (The test hook's stores are counted by vmcnt too, and not in order with the loads, so it always drains.)
  auto wait_loads = [&](bool keep_in_flight) __attribute__((always_inline)) {  // true: the AHEAD-1 youngest stages may stay outstanding
    constexpr int N = LOADS * (AHEAD - 1);
    // s_waitcnt immediate: vmcnt in bits 3:0 and 15:14, expcnt (6:4) and lgkmcnt (11:8) left at "no wait"
    constexpr int KEEP = (N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14), DRAIN = (7 << 4) | (15 << 8);
    if (DUMP || !keep_in_flight || AHEAD == 1) __builtin_amdgcn_s_waitcnt(DRAIN);
    else __builtin_amdgcn_s_waitcnt(KEEP);
    asm volatile("s_barrier" ::: "memory");
  };
  const std::integral_constant<int, SPS> whole_tag;
  const int nwhole = g.K / KC;

  // ---- One software pipeline per wave that runs across the stage barriers.  The unit is the product of one
  // 32x32 sub-block with one quantization block along K: a chain of KPB MFMAs into one INT32 tile, then the
  // fold of that tile into the FP32 accumulator (32 conversions/FMAs; at B = 32 the kernel is bound by them).
  // Two INT32 tiles rotate: the chain of the next unit is issued before the fold of the current one, and at
  // the end of a stage the barrier, the prefetch and the fragment reads of the next stage come BEFORE the fold
  // of the stage's last unit, which covers the LDS latency of those reads.  All fragments of a stage are read
  // at once.
  constexpr int NKB = SPS / KPB;  // quantization blocks along K per stage
  static_assert(SPS % KPB == 0 && (NKB * NTILE) % 2 == 0, "a whole stage leaves the tile rotation where it found it");
  v16i vi[2];
  v4i fa[SPS][WM], fb[SPS][WN];
  // scales two stages ahead of the one in use: requested before a stage barrier, moved one level down at
  // the next, so the scalar loads are never waited for together with LDS fragment reads
  float sa_f[WM][NKB], sb_f[WN][NKB];
#pragma unroll
  for (int j = 0; j < NKB; ++j) {
#pragma unroll
    for (int a = 0; a < WM; ++a) sa_c[a][j] = sa_n[a][j] = sa_f[a][j] = 0.0f;
#pragma unroll
    for (int b = 0; b < WN; ++b) sb_c[b][j] = sb_n[b][j] = sb_f[b][j] = 0.0f;
  }
  // Stages are numbered t = t0 .. tl.  When K is not a multiple of KC the odd K steps (whole quantization
  // blocks) come FIRST, as stage t = -1 in ring slot NBUF-1, so that every stage inside the loops is whole;
  // stage t >= 0 starts at K offset kbase + t*KC and lives in ring slot t % NBUF.
  const int rem = nsteps % SPS, kbase = 32 * rem;
  const int t0 = rem ? -1 : 0, tl = nwhole - 1;
  // Running scalar pointers to the scales of the next stage to request: one 64-bit add per stage and
  // operand sub-tile instead of an index computation per load.
  const_f32_ptr pa[WM], pb[WN];
#pragma unroll
  for (int a = 0; a < WM; ++a) pa[a] = SAc + sa_row[a];
#pragma unroll
  for (int b = 0; b < WN; ++b) pb[b] = SBc + sb_row[b];
  // current <- next <- far <- scalar loads of `blocks` quantization blocks along K (the rest of a stage keeps
  // stale values that are never used); nothing is requested when the far stage does not exist
  auto advance_scales = [&](auto far_exists, int blocks) __attribute__((always_inline)) {
    rotate_scales();
#pragma unroll
    for (int j = 0; j < NKB; ++j) {
#pragma unroll
      for (int a = 0; a < WM; ++a) sa_n[a][j] = sa_f[a][j];
#pragma unroll
      for (int b = 0; b < WN; ++b) sb_n[b][j] = sb_f[b][j];
    }
    if (DUMP) return;
    if (far_exists) {
#pragma unroll
      for (int j = 0; j < NKB; ++j) {
        if (j < blocks) {
#pragma unroll
          for (int a = 0; a < WM; ++a) sa_f[a][j] = pa[a][j * g.sa_k];
#pragma unroll
          for (int b = 0; b < WN; ++b) sb_f[b][j] = pb[b][j * g.sb_k];
        }
      }
#pragma unroll
      for (int a = 0; a < WM; ++a) pa[a] += blocks * g.sa_k;
#pragma unroll
      for (int b = 0; b < WN; ++b) pb[b] += blocks * g.sb_k;
    }
  };
  // stages t >= 0 are whole by construction
  auto issue = [&](int t, int slot) __attribute__((always_inline)) { issue_at(max(0, 32 * (nsteps % SPS) + t * KC), slot, false); };
  auto issue_whole = [&](int t, int slot) __attribute__((always_inline)) { issue_at(32 * (nsteps % SPS) + t * KC, slot, std::true_type()); };
  auto read_frags = [&](int buf) __attribute__((always_inline)) {
    const int8_t* ta = tile_buf(buf);
    const int8_t* tb = ta + A_BYTES;
#pragma unroll
    for (int j = 0; j < SPS; ++j) {
#pragma unroll
      for (int a = 0; a < WM; ++a) fa[j][a] = addrA.read(ta, a, j);
#pragma unroll
      for (int b = 0; b < WN; ++b) fb[j][b] = addrB.read(tb, b, j);
    }
  };
  auto k0_of = [&](int t) __attribute__((always_inline)) { return max(0, kbase + t * KC); };
  auto slot_of = [&](int t) __attribute__((always_inline)) { return (t + NBUF) % NBUF; };
  // registers [16*part/KPB, 16*(part+1)/KPB) of one unit's fold (the test hook stores the whole tile at part 0)
  auto fold_or_dump = [&](int t, int kb, int a, int b, const v16i& v, float scale, auto part_tag) __attribute__((always_inline)) {
    constexpr int part = decltype(part_tag)::value, NPART = KPB;
    if (DUMP) {
      if (part == 0 && k0_of(t) / B + kb == g.dump_kb) dump_tile(v, a, b);
    } else {
      fold<16 * part / NPART, 16 * (part + 1) / NPART>(acc[a][b], v, scale);
    }
  };
  // MFMA number js of the chain of unit i of a stage (quantization block i / NTILE, sub-block i % NTILE) into dst
  auto chain_step = [&](int i, int js, v16i& dst) __attribute__((always_inline)) {
    const int kb = i / NTILE, a = (i % NTILE) / WN, b = (i % NTILE) % WN;
    dst = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[kb * KPB + js][b], fa[kb * KPB + js][a], js == 0 ? zero16 : dst, 0, 0, 0);
  };
  auto chain = [&](int i, v16i& dst) __attribute__((always_inline)) {
#pragma unroll
    for (int js = 0; js < KPB; ++js) chain_step(i, js, dst);
  };
  // One unit's fold with the next unit's chain woven in: each MFMA (32 cycles of the matrix pipe) is followed
  // by 32/KPB vector instructions (4 cycles each), so a single wave keeps both pipes busy and never waits to
  // issue the next MFMA of a chain.  next < 0: fold only.
  auto fold_and_chain = [&](int t, int kb, int a, int b, v16i& cur, float scale, int next, v16i& nxt) __attribute__((always_inline)) {
    static_for<0, KPB>([&](auto js) __attribute__((always_inline)) {
      if (next >= 0) chain_step(next, decltype(js)::value, nxt);
      __builtin_amdgcn_sched_barrier(0);
      fold_or_dump(t, kb, a, b, cur, scale, js);
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  // Stage t out of ring slot `slot`; on entry the chain of its first unit is in flight in vi[0].  With a next
  // stage (in slot `nslot`) the chain of that stage's first unit is in flight in vi[0] on return.
  //   keep: stage t + AHEAD exists (its loads may stay in flight over the barrier);
  //   more: stage t + 1 + AHEAD exists and is prefetched into the slot this stage frees;
  //   far:  stage t + 3 exists (its scales are requested now).
  // The flags are compile-time constants everywhere but in the odd first stage.
  auto run_stage = [&](int t, int slot, int nslot, auto steps_tag, auto has_next, auto keep, auto more, auto far) __attribute__((always_inline)) {
    constexpr int NT = (decltype(steps_tag)::value / KPB) * NTILE;
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      const int kb = i / NTILE, a = (i % NTILE) / WN, b = (i % NTILE) % WN, cur = i & 1;
      const float scale = sa_c[a][kb] * sb_c[b][kb];
      if (i + 1 < NT) {
        fold_and_chain(t, kb, a, b, vi[cur], scale, i + 1, vi[cur ^ 1]);
      } else if (has_next) {
        advance_scales(far, NKB);  // before the barrier: the wait there covers the scalar loads
        wait_loads(keep);
        if (more) issue_whole(t + 1 + AHEAD, slot);
        read_frags(nslot);
        fold_and_chain(t, kb, a, b, vi[cur], scale, -1, vi[cur]);
        chain(0, vi[0]);
      } else {
        fold_and_chain(t, kb, a, b, vi[cur], scale, -1, vi[cur]);
      }
    }
  };

  static_assert(NBUF >= 3, "a prefetched stage implies the stage whose scales are requested");
  // the tiles of the first stages are requested before the scales: the second scale request waits for the first
#pragma unroll
  for (int i = 0; i < AHEAD; ++i)
    if (t0 + i <= tl) issue(t0 + i, slot_of(t0 + i));
  advance_scales(true, (rem ? rem : SPS) / KPB);
  advance_scales(t0 + 1 <= tl, NKB);
  wait_loads(t0 + AHEAD - 1 <= tl);
  if (t0 + AHEAD <= tl) issue(t0 + AHEAD, slot_of(t0 + AHEAD));
  advance_scales(t0 + 2 <= tl, NKB);
  read_frags(slot_of(t0));
  chain(0, vi[0]);
  if (rem) {  // the odd first stage: 1 .. SPS-1 K steps, an odd tile count flips the rotation, hence vi[0] again
    const bool has_next = tl >= 0, keep = AHEAD - 1 <= tl, more = AHEAD <= tl, far = 2 <= tl;
    if constexpr (SPS >= 2 && KPB == 1) { if (rem == 1) run_stage(-1, NBUF - 1, 0, std::integral_constant<int, 1>(), has_next, keep, more, far); }
    if constexpr (SPS >= 4 && KPB <= 2) { if (rem == 2) run_stage(-1, NBUF - 1, 0, std::integral_constant<int, 2>(), has_next, keep, more, far); }
    if constexpr (SPS >= 4 && KPB == 1) { if (rem == 3) run_stage(-1, NBUF - 1, 0, std::integral_constant<int, 3>(), has_next, keep, more, far); }
  }
  // Main loop: passes of NBUF whole stages, each with a successor and a stage to prefetch, so the ring slot
  // of every stage is a compile-time constant: LDS addresses are immediates and the accumulators never move.
  int t = 0;
  for (; t + 2 * NBUF - 1 <= tl; t += NBUF) {
    // The instruction arbiter favours the oldest wave of a SIMD, so co-resident waves would finish one after
    // the other and leave the SIMD to a single wave at the end.  Each wave therefore lowers its own priority
    // as it advances: whoever is ahead yields, and the waves of a SIMD reach the end together.
    if (4 * t < nstages) __builtin_amdgcn_s_setprio(3);
    else if (2 * t < nstages) __builtin_amdgcn_s_setprio(2);
    else if (4 * t < 3 * nstages) __builtin_amdgcn_s_setprio(1);
    else __builtin_amdgcn_s_setprio(0);
#pragma unroll
    for (int u = 0; u < NBUF; ++u)
      run_stage(t + u, u, (u + 1) % NBUF, whole_tag, std::true_type(), std::true_type(), std::true_type(), std::true_type());
  }
  // The last R = 1 .. 2*NBUF-1 stages as straight-line code per R, so that their flags are constants too.
  __builtin_amdgcn_s_setprio(0);
  auto run_tail = [&](auto r_tag) __attribute__((always_inline)) {
    constexpr int R = decltype(r_tag)::value;
    static_for<0, R>([&](auto i_tag) __attribute__((always_inline)) {
      constexpr int i = decltype(i_tag)::value;
      run_stage(t + i, i % NBUF, (i + 1) % NBUF, whole_tag, std::integral_constant<bool, (i + 1 < R)>(),
                std::integral_constant<bool, (i + AHEAD < R)>(), std::integral_constant<bool, (i + 1 + AHEAD < R)>(),
                std::integral_constant<bool, (i + 3 < R)>());
    });
  };
  const int R = tl - t + 1;
  static_for<1, 2 * NBUF>([&](auto r_tag) __attribute__((always_inline)) {
    if (R == decltype(r_tag)::value) run_tail(r_tag);
  });
  if (DUMP) return;

  // ---- epilogue: optional FP32 store, per-block max-abs, Eq. 1, packed INT8 store
  float amax[WM][WN];
#pragma unroll
  for (int a = 0; a < WM; ++a)
#pragma unroll
    for (int b = 0; b < WN; ++b) {
      float m = 0.0f;
#pragma unroll
      for (int r = 0; r < 16; ++r) m = fmaxf(m, fabsf(acc[a][b][r]));
      amax[a][b] = wave_group_max<63>(m);
    }
  if (B > 32) {
    if (lane == 0) {
#pragma unroll
      for (int a = 0; a < WM; ++a)
#pragma unroll
        for (int b = 0; b < WN; ++b) s_amax[wm0 + a][wn0 + b] = amax[a][b];
    }
    __syncthreads();
    constexpr int G = B / 32;
#pragma unroll
    for (int a = 0; a < WM; ++a)
#pragma unroll
      for (int b = 0; b < WN; ++b) {
        const int ga = ((wm0 + a) / G) * G, gb = ((wn0 + b) / G) * G;
        float m = 0.0f;
        for (int x = 0; x < G; ++x)
          for (int y = 0; y < G; ++y) m = fmaxf(m, s_amax[ga + x][gb + y]);
        amax[a][b] = m;
      }
  }
  const int ln = g.Nn / B;
  // The code tile is staged in the operand ring: in one slot, or split by rows over two slots when a slot is
  // smaller than the tile.  The last stage of the K loop ends without a barrier, so a wave may still be reading its
  // fragments of that stage out of the ring while a faster one is already here: meet once before the ring is
  // overwritten (for B > 32 the barrier of the max-abs exchange above has done that).
  if (B == 32 && g.Oq != nullptr) __syncthreads();
  constexpr int CODE_ROWS_PER_SLOT = TM * TN <= STAGE_BYTES ? TM : TM / 2;
  static_assert(CODE_ROWS_PER_SLOT * TN <= STAGE_BYTES, "half the code tile fits a ring slot");
  auto code_row = [&](int row) __attribute__((always_inline)) -> int8_t* {
    return (row < CODE_ROWS_PER_SLOT ? s_tile0 : s_tile1) + (row % CODE_ROWS_PER_SLOT) * TN;
  };
#pragma unroll
  for (int a = 0; a < WM; ++a)
#pragma unroll
    for (int b = 0; b < WN; ++b) {
      const int mrow0 = m0 + 32 * (wm0 + a), ncol0 = n0 + 32 * (wn0 + b);
      if (mrow0 >= g.M || ncol0 >= g.Nn) continue;  // wave-uniform: the whole sub-block is outside
      const int m = mrow0 + (lane & 31);
      const int nb = ncol0 + 4 * (lane >> 5);
      if (g.Of) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
          *reinterpret_cast<float4*>(g.Of + (int64_t)m * g.Nn + nb + 8 * q4) =
              make_float4(acc[a][b][4 * q4], acc[a][b][4 * q4 + 1], acc[a][b][4 * q4 + 2], acc[a][b][4 * q4 + 3]);
      }
      if (g.Oq) {
        float scale;
        double inv;
        block_scale(amax[a][b], scale, inv);
        if (lane == 0 && (mrow0 % B) == 0 && (ncol0 % B) == 0) g.Os[(int64_t)(mrow0 / B) * ln + ncol0 / B] = scale;
        // Codes go to LDS first, laid out as the TM x TN byte tile with its 16-byte chunks XOR-swizzled by the
        // row, so that the tile can be written to memory as whole rows.
        const int row = 32 * (wm0 + a) + (lane & 31);
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int col = 32 * (wn0 + b) + 8 * q4 + 4 * (lane >> 5);
          const int chunk = (col >> 4) ^ (row & (TN / 16 - 1));
          *reinterpret_cast<uint32_t*>(code_row(row) + 16 * chunk + (col & 15)) =
              quantize4(acc[a][b][4 * q4], acc[a][b][4 * q4 + 1], acc[a][b][4 * q4 + 2], acc[a][b][4 * q4 + 3], inv);
        }
      }
    }
  if (g.Oq) {
    // TN / 16 consecutive lanes write one TN-byte row of the tile: full 128-byte lines for the 128-wide tile.
    __syncthreads();
    constexpr int CPRO = TN / 16;
    static_assert((TM * CPRO) % (64 * NW) == 0, "whole passes over the code tile");
#pragma unroll
    for (int i = 0; i < (TM * CPRO) / (64 * NW); ++i) {
      const int id = i * 64 * NW + tid;
      const int row = id / CPRO, c = id % CPRO;
      if (m0 + row < g.M && n0 + 16 * c < g.Nn) {
        const uint4 v = *reinterpret_cast<const uint4*>(code_row(row) + 16 * (c ^ (row & (CPRO - 1))));
        *reinterpret_cast<uint4*>(g.Oq + (int64_t)(m0 + row) * g.Nn + n0 + 16 * c) = v;
      }
    }
  }
}

// One product per launch.  WMIN = minimum resident waves per SIMD the register allocation must allow.
template <int B, int WM, int WN, int WGM, int WGN, bool AK, bool BK, bool DUMP, int WMIN, bool DEEP = false>
__global__ void __launch_bounds__(64 * WGM * WGN, WMIN) gemm_kernel(const GemmArgs g) {
  typedef GemmShape<B, WM, WN, WGM, WGN, AK, BK, DEEP> Shape;
  __shared__ __align__(1024) int8_t s_ring[Shape::RING_BYTES];
  __shared__ float s_amax[8][8];
  gemm_tile<B, WM, WN, WGM, WGN, AK, BK, DUMP, DEEP>(g, blockIdx.x, gridDim.x, s_ring, s_amax);
}

// Two independent products in one launch -- the input gradient and the weight gradient of a layer (Sec. 4), which
// need the same dY and nothing of each other.  Workgroups 0 .. tiles_first - 1 take tiles of the first product, the
// others of the second; both use four-wave workgroups, so the ring is the larger of the two.  Each product alone
// has too few tiles to keep the chip busy to the end, and pays its own ramp-up, first-stage latency and epilogue;
// in one launch the scheduler starts tiles of the second as those of the first finish, so that those phases of
// some workgroups run beside the K loops of others.
template <class First, class Second, int WMIN>
__global__ void __launch_bounds__(256, WMIN) gemm_pair_kernel(const GemmArgs g1, const GemmArgs g2, const int tiles_first) {
  constexpr int RING = First::Shape::RING_BYTES > Second::Shape::RING_BYTES ? First::Shape::RING_BYTES : Second::Shape::RING_BYTES;
  __shared__ __align__(1024) int8_t s_ring[RING];
  __shared__ float s_amax[8][8];
  if ((int)blockIdx.x < tiles_first) First::run(g1, blockIdx.x, tiles_first, s_ring, s_amax);
  else Second::run(g2, blockIdx.x - tiles_first, gridDim.x - tiles_first, s_ring, s_amax);
}
// a product's instance as a type, for gemm_pair_kernel
template <int B, int WM, int WN, int WGM, int WGN, bool AK, bool BK, bool DEEP>
struct GemmInstance {
  typedef GemmShape<B, WM, WN, WGM, WGN, AK, BK, DEEP> Shape;
  static_assert(Shape::NW == 4, "pairs are built from four-wave workgroups");
  static __device__ __forceinline__ void run(const GemmArgs& g, int tile_index, int ntiles, int8_t* s_ring, float (*s_amax)[8]) {
    gemm_tile<B, WM, WN, WGM, WGN, AK, BK, false, DEEP>(g, tile_index, ntiles, s_ring, s_amax);
  }
  static int tiles(const GemmArgs& a) { return ((a.M + Shape::TM - 1) / Shape::TM) * ((a.Nn + Shape::TN - 1) / Shape::TN); }
};

// --------------------------------------------------------------------- host
template <int B, int WM, int WN, int WGM, int WGN, bool AK, bool BK, bool DUMP, bool DEEP = false>
static void launch_cfg(const GemmArgs& a, hipStream_t st) {
  constexpr int TM = 32 * WM * WGM, TN = 32 * WN * WGN;
  // resident waves per SIMD the register allocation has to allow: 3 for the 2x2 wave tile (three
  // 128x128 workgroups share a compute unit), the waves of the one workgroup per compute unit for the big
  // workgroups (2 for eight waves, 3 for nine or twelve), 4 for the 64x64 tiles
  // (3 for the 64x64 tiles with a stage of 128 K bytes: their ring leaves room for three workgroups per compute unit)
  constexpr int WMIN = (WM * WN >= 4 && WGM * WGN == 8) ? 2 : (WM * WN >= 4) ? 3 : (WGM * WGN > 8 ? 3 : (WGM * WGN > 4 ? 2 : ((DEEP || B == 64) ? 3 : 4)));
  const int tiles = ((a.M + TM - 1) / TM) * ((a.Nn + TN - 1) / TN);
  hipLaunchKernelGGL((gemm_kernel<B, WM, WN, WGM, WGN, AK, BK, DUMP, WMIN, DEEP>), dim3(tiles), dim3(64 * WGM * WGN), 0, st, a);
}

// Tile shapes.  At B = 32 the kernel is bound by the vector ALU work of the per-K-block dequantization, which
// is the same per output element for every shape; what differs is what a wave pays per MFMA for fragment reads and
// staging (less for the larger wave tiles), how evenly the tiles fill 256 compute units, and the fixed cost of a
// tile.  Four-wave workgroups throughout:
//   128x128  waves of 2x2 sub-blocks, three workgroups per compute unit;
//   128x64   waves of 2x1 sub-blocks, four workgroups per compute unit;
//    64x64   waves of one sub-block, four per compute unit; with a stage of 128 instead of 64 K bytes (half the
//            barriers, three workgroups per compute unit) when the output has at most 768 such tiles and one operand
//            is K-major.
// The shape is chosen by a model of the busiest SIMD, fitted to the measured times of 39 products (the layers of the
// benchmark configurations, 9 us to 180 us, all three operand layouts): a workgroup puts one wave of `sub` sub-blocks
// on every SIMD of its compute unit; with T tiles the busiest unit holds ceil(T / 256) workgroups while they are all
// resident at once, T / 256 + tail beyond that; a sub-block and K step costs `ns` on a SIMD that holds at least two
// waves and `ns_alone` on one that holds a single wave (which cannot overlap its own MFMA and fold); `fixed_us` is
// the launch, first-stage latency and epilogue.  On those 39 products the model's choice is within 0.2 % of the best
// shape in total (8 % at worst).
extern std::atomic<int> g_forced_shape;  // test hook, see jf_debug_set_gemm_shape: 0 unless a test sets it
struct ShapeModel {
  int tm, tn, sub, resident;
  double fixed_us, ns, ns_alone, tail;
};
static double shape_cost_us(const ShapeModel& m, const GemmArgs& a) {
  const double tiles = (double)((a.M + m.tm - 1) / m.tm) * ((a.Nn + m.tn - 1) / m.tn);
  const double per_cu = tiles / 256.0;
  const double busiest = tiles <= 256.0 * m.resident ? std::ceil(per_cu) : per_cu + m.tail;
  return m.fixed_us + busiest * m.sub * (a.K / 32) * (busiest <= 1.0 ? m.ns_alone : m.ns) * 1e-3;
}
static const ShapeModel kShape128x128 = {128, 128, 4, 3, 6.5, 61.0, 88.0, 0.5};
static const ShapeModel kShape128x64 = {128, 64, 2, 4, 4.5, 69.0, 112.0, 0.75};
static const ShapeModel kShape64x64 = {64, 64, 1, 4, 4.0, 82.0, 172.0, 0.75};
// Tile shape of a block-32 product, numbered as in jf_debug_set_gemm_shape: 1 128x128, 4 64x64, 7 64x64 with a
// stage of 128 K bytes, 8 128x64.
template <bool AK, bool BK>
static int choose_shape_b32(const GemmArgs& a) {
  const int forced = g_forced_shape.load(std::memory_order_relaxed);
  if (forced == 1 || forced == 4 || forced == 7 || forced == 8) return forced;
  const double c1 = shape_cost_us(kShape128x128, a), c8 = shape_cost_us(kShape128x64, a), c4 = shape_cost_us(kShape64x64, a);
  if (c1 <= c8 && c1 <= c4) return 1;
  if (c8 <= c4) return 8;
  const int64_t n64 = (int64_t)((a.M + 63) / 64) * ((a.Nn + 63) / 64);
  return ((AK || BK) && n64 <= 768) ? 7 : 4;
}

template <int B, bool AK, bool BK, bool DUMP>
static void launch_shape(const GemmArgs& a, hipStream_t st) {
  const int g_forced_shape = jf::g_forced_shape.load(std::memory_order_relaxed);
  if (g_forced_shape == 6) {
    launch_cfg<B, 2, 2, 4, 2, AK, BK, DUMP>(a, st);
    return;
  }
  if constexpr (B == 128) {
    // Eight waves per workgroup, one workgroup per compute unit.  256x128 tile (waves of 2x2 sub-blocks): a
    // third less L2 -> LDS traffic per MFMA, measured 10 % faster on every large shape; outputs with fewer
    // than 256 such tiles take the 128x128 tile (waves of 2x1 sub-blocks) so that every compute unit has work.
    const int64_t big_tiles = (int64_t)((a.M + 255) / 256) * ((a.Nn + 127) / 128);
    if (big_tiles >= 256 && g_forced_shape != 1) launch_cfg<B, 2, 2, 4, 2, AK, BK, DUMP>(a, st);
    else launch_cfg<B, 2, 1, 2, 4, AK, BK, DUMP>(a, st);
  } else if constexpr (B == 64) {
    // 128x128 (waves of 2x2 sub-blocks) or 64x64 (waves of one), by the same model with the constants of this block
    // size (half the fold per MFMA): fitted to the same layer shapes, the choice is within 5 % of the better one.
    static const ShapeModel k128 = {128, 128, 4, 3, 6.5, 44.0, 63.0, 0.5}, k64 = {64, 64, 1, 3, 4.0, 65.0, 190.0, 0.75};
    const bool big = g_forced_shape ? g_forced_shape != 4 : shape_cost_us(k128, a) <= shape_cost_us(k64, a);
    if (big)
      launch_cfg<B, 2, 2, 2, 2, AK, BK, DUMP>(a, st);
    else
      launch_cfg<B, 1, 1, 2, 2, AK, BK, DUMP>(a, st);
  } else {
    const int shape = choose_shape_b32<AK, BK>(a);
    if (shape == 1) launch_cfg<B, 2, 2, 2, 2, AK, BK, DUMP>(a, st);
    else if (shape == 8) launch_cfg<B, 2, 1, 2, 2, AK, BK, DUMP>(a, st);
    else if (shape == 7) launch_cfg<B, 1, 1, 2, 2, AK, BK, DUMP, true>(a, st);
    else launch_cfg<B, 1, 1, 2, 2, AK, BK, DUMP>(a, st);
  }
}

// One translation unit per (product, block size) instantiates this, so that the kernels compile in parallel.
// AK / BK: operand A / Bm is K-major.
template <int B, bool AK, bool BK>
static void launch_product(const GemmArgs& a, bool dump, hipStream_t st) {
  if (dump) launch_shape<B, AK, BK, true>(a, st);
  else launch_shape<B, AK, BK, false>(a, st);
}

#define JF_GEMM_INSTANCE(NAME, B, AK, BK) \
  namespace jf { void NAME(const GemmArgs& a, bool dump, hipStream_t st) { launch_product<B, AK, BK>(a, dump, st); } }

#ifdef JF_GEMM_PAIR_INSTANCES   // defined by the one translation unit that holds the pair kernels
// Input gradient and weight gradient of a block-32 layer in one launch (gemm_pair_kernel), when each of them alone
// would run on 64 x 64 tiles, i.e. has too few tiles for the larger shapes.  The weight gradient's tiles, whose K loop
// over the tokens is the longer one, are dealt first.  Returns false (nothing launched) when the shapes do not suit.
static bool launch_bwd_pair_b32(const GemmArgs& dgrad, const GemmArgs& wgrad, hipStream_t st) {
  typedef GemmInstance<32, 1, 1, 2, 2, false, false, false> Wgrad;
  typedef GemmInstance<32, 1, 1, 2, 2, true, false, false> Dgrad;
  typedef GemmInstance<32, 1, 1, 2, 2, true, false, true> DgradDeep;
  if (g_forced_shape.load(std::memory_order_relaxed) != 0) return false;   // a forced shape means the single-product kernels
  // One grid of 64 x 64 tiles of both products against each product alone on its own best shape, by the model above:
  // in the pair the tiles of the second product fill the compute units that the first leaves idle, so the busiest
  // SIMD works through the average number of sub-blocks (88 ns each with the pair's mix of operand layouts, measured
  // at the GPT-2-small and GPT-2-large layer shapes) and the fixed cost is paid once.
  const double ksd = dgrad.K / 32, ksw = wgrad.K / 32;
  const int tw = Wgrad::tiles(wgrad), td = Dgrad::tiles(dgrad);
  const double pair_us = 5.0 + (td * ksd + tw * ksw) / 256.0 * 88.0e-3;
  double alone_us = 0.0;
  for (const GemmArgs* g : {&dgrad, &wgrad})
    alone_us += std::min(shape_cost_us(kShape128x128, *g), std::min(shape_cost_us(kShape128x64, *g), shape_cost_us(kShape64x64, *g)));
  // (the first part has to be a multiple of 8 workgroups, so that both parts see the same XCD numbering)
  if (pair_us >= alone_us || tw % 8) return false;
  const int sd = ((int64_t)td <= 768) ? 7 : 4;   // the deep stage pays while the tiles of dgrad are resident at once
  if (sd == 7) hipLaunchKernelGGL((gemm_pair_kernel<Wgrad, DgradDeep, 3>), dim3(tw + td), dim3(256), 0, st, wgrad, dgrad, tw);
  else hipLaunchKernelGGL((gemm_pair_kernel<Wgrad, Dgrad, 3>), dim3(tw + td), dim3(256), 0, st, wgrad, dgrad, tw);
  return true;
}
#endif

}  // namespace jf
