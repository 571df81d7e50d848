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

// KC = bytes of K staged per LDS stage: 64 (two MFMA K steps), 128 for B = 128 so that a stage
// always holds whole quantization blocks and block boundaries are known at compile time.
template <int TILE, bool KMAJOR, int KC>
struct TileLayout {
  static constexpr int kRows = KMAJOR ? TILE : KC;
  static constexpr int kStride = (KMAJOR ? KC : TILE) + 16;  // 16 * odd: conflict-free b128 / tr_b64 reads
  static constexpr int kBytes = kRows * kStride;
  static constexpr int kChunks = TILE * KC / 16;             // 16-byte chunks per stage
};

// Copy description of one 16-byte chunk c of a stage: where it comes from and where it lands in LDS.
template <int TILE, bool KMAJOR, int KC>
__device__ __forceinline__ void chunk_coords(int c, int& outer, int& kk, int& lds_off) {
  if (KMAJOR) {
    const int row = c / (KC / 16), kc = c % (KC / 16);
    outer = row;
    kk = 16 * kc;
    lds_off = row * TileLayout<TILE, true, KC>::kStride + 16 * kc;
  } else {
    const int krow = c / (TILE / 16), mc = c % (TILE / 16);
    outer = 16 * mc;
    kk = krow;
    lds_off = krow * TileLayout<TILE, false, KC>::kStride + 16 * mc;
  }
}

// One MFMA operand fragment (16 bytes of K for row lane%32) of the 32-row sub-tile `sub`, K step j of the stage.
template <int TILE, bool KMAJOR, int KC>
__device__ __forceinline__ v4i read_frag(const int8_t* tile, int sub, int j, int lane) {
  typedef __attribute__((address_space(3))) v2i* lds_v2i;
  if (KMAJOR) {
    const int8_t* p = tile + (sub * 32 + (lane & 31)) * TileLayout<TILE, true, KC>::kStride + j * 32 + 16 * (lane >> 5);
    return *reinterpret_cast<const v4i*>(p);
  } else {
    // ds_read_b64_tr_b8: within 16 lanes, lane 2r+h points at 8 bytes (columns 8h..8h+7) of row r;
    // lane c receives column c of that 8 x 16 byte matrix.
    const int i = lane & 15, g = lane >> 4;
    const int krow = j * 32 + 16 * (g >> 1) + (i >> 1);
    const int mcol = sub * 32 + 16 * (g & 1) + 8 * (i & 1);
    const int8_t* p = tile + krow * TileLayout<TILE, false, KC>::kStride + mcol;
    v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i)(p));
    v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((lds_v2i)(p + 8 * TileLayout<TILE, false, KC>::kStride));
    v4i r = {lo[0], lo[1], hi[0], hi[1]};
    return r;
  }
}

template <int B, int WM, int WN, int WGM, int WGN, bool AK, bool BK, bool DUMP>
__global__ void __launch_bounds__(64 * WGM * WGN, 2) gemm_kernel(const GemmArgs g) {
  constexpr int NT = 64 * WGM * WGN;
  constexpr int TM = 32 * WM * WGM, TN = 32 * WN * WGN;
  constexpr int KPB = B / 32;  // MFMA K steps per quantization block
  constexpr int KC = B == 128 ? 128 : 64;
  constexpr int SPS = KC / 32;  // MFMA K steps per stage
  typedef TileLayout<TM, AK, KC> LA;
  typedef TileLayout<TN, BK, KC> LB;
  constexpr int CA = (LA::kChunks + NT - 1) / NT, CB = (LB::kChunks + NT - 1) / NT;
  constexpr int NSA = (TM / 32) * SPS, NSB = (TN / 32) * SPS;  // scales staged per stage: [32-row granule][K step]
  static_assert(B == 32 || (TM % B == 0 && TN % B == 0), "tile must hold whole quantization blocks");
  static_assert(NSA + NSB <= NT, "one scale per thread");

  __shared__ __align__(16) int8_t s_tiles[2][LA::kBytes + LB::kBytes];
  __shared__ float s_scales[2][NSA + NSB];
  __shared__ float s_amax[TM / 32][TN / 32];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave / WGN) * WM, wn0 = (wave % WGN) * WN;  // first 32-granule of this wave inside the tile
  const int tiles_n = (g.Nn + TN - 1) / TN;
  const int m0 = (blockIdx.x / tiles_n) * TM, n0 = (blockIdx.x % tiles_n) * TN;

  v4i pa[CA], pb[CB];
  float psc = 0.0f;

  auto gload = [&](int k0) {
#pragma unroll
    for (int i = 0; i < CA; ++i) {
      const int c = tid + i * NT;
      int outer, kk, off;
      chunk_coords<TM, AK, KC>(c, outer, kk, off);
      const bool ok = (LA::kChunks % NT == 0 || c < LA::kChunks) && (m0 + outer < g.M) && (k0 + kk < g.K);
      const int8_t* p = AK ? g.A + (int64_t)(m0 + outer) * g.lda + (k0 + kk) : g.A + (int64_t)(k0 + kk) * g.lda + (m0 + outer);
      v4i z = {0, 0, 0, 0};
      pa[i] = ok ? *reinterpret_cast<const v4i*>(p) : z;
    }
#pragma unroll
    for (int i = 0; i < CB; ++i) {
      const int c = tid + i * NT;
      int outer, kk, off;
      chunk_coords<TN, BK, KC>(c, outer, kk, off);
      const bool ok = (LB::kChunks % NT == 0 || c < LB::kChunks) && (n0 + outer < g.Nn) && (k0 + kk < g.K);
      const int8_t* p = BK ? g.Bm + (int64_t)(n0 + outer) * g.ldb + (k0 + kk) : g.Bm + (int64_t)(k0 + kk) * g.ldb + (n0 + outer);
      v4i z = {0, 0, 0, 0};
      pb[i] = ok ? *reinterpret_cast<const v4i*>(p) : z;
    }
    if (!DUMP && tid < NSA + NSB) {
      const bool isA = tid < NSA;
      const int e = isA ? tid : tid - NSA;
      const int gr = (isA ? m0 : n0) + 32 * (e / SPS), gk = k0 + 32 * (e % SPS);
      const bool ok = gr < (isA ? g.M : g.Nn) && gk < g.K;
      const float* S = isA ? g.SA : g.SB;
      const int sp = isA ? g.sa_p : g.sb_p, sk = isA ? g.sa_k : g.sb_k;
      psc = ok ? S[(int64_t)(gr / B) * sp + (int64_t)(gk / B) * sk] : 0.0f;
    }
  };
  auto lstore = [&](int buf) {
    int8_t* ta = s_tiles[buf];
    int8_t* tb = ta + LA::kBytes;
#pragma unroll
    for (int i = 0; i < CA; ++i) {
      const int c = tid + i * NT;
      int outer, kk, off;
      chunk_coords<TM, AK, KC>(c, outer, kk, off);
      if (LA::kChunks % NT == 0 || c < LA::kChunks) *reinterpret_cast<v4i*>(ta + off) = pa[i];
    }
#pragma unroll
    for (int i = 0; i < CB; ++i) {
      const int c = tid + i * NT;
      int outer, kk, off;
      chunk_coords<TN, BK, KC>(c, outer, kk, off);
      if (LB::kChunks % NT == 0 || c < LB::kChunks) *reinterpret_cast<v4i*>(tb + off) = pb[i];
    }
    if (!DUMP && tid < NSA + NSB) s_scales[buf][tid] = psc;
  };

  float acc[WM][WN][16];
  v16i vi[WM][WN];
  const v16i zero16 = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int a = 0; a < WM; ++a)
#pragma unroll
    for (int b = 0; b < WN; ++b) {
      vi[a][b] = zero16;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;
    }

  const int nsteps = g.K / 32;
  const int nstages = (g.K + KC - 1) / KC;
  gload(0);
  lstore(0);
  __syncthreads();
  for (int s = 0; s < nstages; ++s) {
    const int buf = s & 1;
    if (s + 1 < nstages) gload((s + 1) * KC);
    const int8_t* ta = s_tiles[buf];
    const int8_t* tb = ta + LA::kBytes;
#pragma unroll
    for (int j = 0; j < SPS; ++j) {
      const int step = s * SPS + j;
      if (step < nsteps) {
        v4i fa[WM], fb[WN];
#pragma unroll
        for (int a = 0; a < WM; ++a) fa[a] = read_frag<TM, AK, KC>(ta, wm0 + a, j, lane);
#pragma unroll
        for (int b = 0; b < WN; ++b) fb[b] = read_frag<TN, BK, KC>(tb, wn0 + b, j, lane);
#pragma unroll
        for (int a = 0; a < WM; ++a)
#pragma unroll
          for (int b = 0; b < WN; ++b)
            vi[a][b] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[b], fa[a], (j % KPB == 0) ? zero16 : vi[a][b], 0, 0, 0);
        if ((j + 1) % KPB == 0) {  // end of a quantization block along K (a stage holds whole blocks)
          if (DUMP) {
            if (step / KPB == g.dump_kb) {
#pragma unroll
              for (int a = 0; a < WM; ++a)
#pragma unroll
                for (int b = 0; b < WN; ++b) {
                  const int m = m0 + 32 * (wm0 + a) + (lane & 31);
                  const int nb = n0 + 32 * (wn0 + b) + 4 * (lane >> 5);
                  if (m < g.M && nb < g.Nn) {
#pragma unroll
                    for (int q4 = 0; q4 < 4; ++q4) {
                      v4i o = {vi[a][b][4 * q4], vi[a][b][4 * q4 + 1], vi[a][b][4 * q4 + 2], vi[a][b][4 * q4 + 3]};
                      *reinterpret_cast<v4i*>(g.dump + (int64_t)m * g.Nn + nb + 8 * q4) = o;
                    }
                  }
                }
            }
          } else {
            float sa[WM], sb[WN];
#pragma unroll
            for (int a = 0; a < WM; ++a) sa[a] = s_scales[buf][(wm0 + a) * SPS + j];
#pragma unroll
            for (int b = 0; b < WN; ++b) sb[b] = s_scales[buf][NSA + (wn0 + b) * SPS + j];
#pragma unroll
            for (int a = 0; a < WM; ++a)
#pragma unroll
              for (int b = 0; b < WN; ++b) {
                const float t = sa[a] * sb[b];
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[a][b][r] = __builtin_fmaf(t, (float)vi[a][b][r], acc[a][b][r]);
              }
          }
        }
      }
    }
    if (s + 1 < nstages) lstore(buf ^ 1);
    __syncthreads();
  }
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
        float scale, inv;
        block_scale(amax[a][b], scale, inv);
        if (lane == 0 && (mrow0 % B) == 0 && (ncol0 % B) == 0) g.Os[(int64_t)(mrow0 / B) * ln + ncol0 / B] = scale;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
          *reinterpret_cast<uint32_t*>(g.Oq + (int64_t)m * g.Nn + nb + 8 * q4) =
              quantize4(acc[a][b][4 * q4], acc[a][b][4 * q4 + 1], acc[a][b][4 * q4 + 2], acc[a][b][4 * q4 + 3], inv);
      }
    }
}

// --------------------------------------------------------------------- host
template <int B, int WM, int WN, int WGM, int WGN, bool AK, bool BK, bool DUMP>
static void launch_cfg(const GemmArgs& a, hipStream_t st) {
  constexpr int TM = 32 * WM * WGM, TN = 32 * WN * WGN;
  const int tiles = ((a.M + TM - 1) / TM) * ((a.Nn + TN - 1) / TN);
  hipLaunchKernelGGL((gemm_kernel<B, WM, WN, WGM, WGN, AK, BK, DUMP>), dim3(tiles), dim3(64 * WGM * WGN), 0, st, a);
}

// Two tile shapes: 128x128 (each wave 2x2 sub-blocks) and 64x64 (each wave one sub-block).  The INT8 path is
// bound by the vector ALU work of the per-K-block dequantization, which is the same per output element for
// every tile shape, so the shape is chosen for an even spread of that work over the 256 compute units.
template <int B, bool AK, bool BK, bool DUMP>
static void launch_shape(const GemmArgs& a, hipStream_t st) {
  auto rounds = [&](int tm, int tn) {
    const int64_t tiles = (int64_t)((a.M + tm - 1) / tm) * ((a.Nn + tn - 1) / tn);
    return (tiles + 255) / 256 * (int64_t)(tm / 32) * (tn / 32);
  };
  if constexpr (B == 128) {
    launch_cfg<B, 2, 2, 2, 2, AK, BK, DUMP>(a, st);
  } else {
    if (rounds(128, 128) <= rounds(64, 64))
      launch_cfg<B, 2, 2, 2, 2, AK, BK, DUMP>(a, st);
    else
      launch_cfg<B, 1, 1, 2, 2, AK, BK, DUMP>(a, st);
  }
}

template <bool AK, bool BK, bool DUMP>
static void launch_block(int block, const GemmArgs& a, hipStream_t st) {
  if (block == 32) launch_shape<32, AK, BK, DUMP>(a, st);
  else if (block == 64) launch_shape<64, AK, BK, DUMP>(a, st);
  else launch_shape<128, AK, BK, DUMP>(a, st);
}

// which: 0 forward, 1 dgrad, 2 wgrad
static void launch_gemm(int which, int block, const GemmArgs& a, bool dump, hipStream_t st) {
  if (which == 0) dump ? launch_block<true, true, true>(block, a, st) : launch_block<true, true, false>(block, a, st);
  else if (which == 1) dump ? launch_block<true, false, true>(block, a, st) : launch_block<true, false, false>(block, a, st);
  else dump ? launch_block<false, false, true>(block, a, st) : launch_block<false, false, false>(block, a, st);
}

static int32_t check_linear(const void* p0, const void* p1, const void* p2, const void* p3, int64_t N, int64_t C,
                            int64_t D, int32_t block) {
  if (!p0 || !p1 || !p2 || !p3) return JF_ERR_NULL;
  if (!valid_block(block)) return JF_ERR_BLOCK;
  if (!valid_dim(N, block) || !valid_dim(C, block) || !valid_dim(D, block)) return JF_ERR_SHAPE;
  if (!aligned16(p0) || !aligned4(p1) || !aligned16(p2) || !aligned4(p3)) return JF_ERR_ALIGN;
  return JF_OK;
}

static int32_t check_out(const int8_t* q, const float* s, const float* f, bool q_required) {
  if ((q == nullptr) != (s == nullptr)) return JF_ERR_NULL;
  if (q_required && !q) return JF_ERR_NULL;
  if (!q && !f) return JF_ERR_NULL;
  if ((q && !aligned16(q)) || (s && !aligned4(s)) || (f && !aligned16(f))) return JF_ERR_ALIGN;
  return JF_OK;
}

// Operand description of the three products in the canonical out = A Bm^T form.
static GemmArgs make_args(int which, const int8_t* a, const float* sa, const int8_t* b, const float* sb, int64_t N,
                          int64_t C, int64_t D, int32_t block) {
  GemmArgs g{};
  g.A = a; g.SA = sa; g.Bm = b; g.SB = sb;
  const int LN = (int)(N / block), LC = (int)(C / block), LD = (int)(D / block);
  (void)LN;
  if (which == 0) {         // Y = X W^T : A = X (N x C) K-major, Bm = W (D x C) K-major
    g.M = (int)N; g.Nn = (int)D; g.K = (int)C; g.lda = C; g.ldb = C;
    g.sa_p = LC; g.sa_k = 1; g.sb_p = LC; g.sb_k = 1;
  } else if (which == 1) {  // dX = dY W : A = dY (N x D) K-major, Bm = W^T stored as W (D x C) = K rows x Nn
    g.M = (int)N; g.Nn = (int)C; g.K = (int)D; g.lda = D; g.ldb = C;
    g.sa_p = LD; g.sa_k = 1; g.sb_p = 1; g.sb_k = LC;
  } else {                  // dW = dY^T X : A = dY^T stored as dY (N x D), Bm = X^T stored as X (N x C)
    g.M = (int)D; g.Nn = (int)C; g.K = (int)N; g.lda = D; g.ldb = C;
    g.sa_p = 1; g.sa_k = LD; g.sb_p = 1; g.sb_k = LC;
  }
  return g;
}

}  // namespace jf

extern "C" int32_t jf_linear_fwd(const int8_t* X, const float* SX, const int8_t* W, const float* SW, int64_t N,
                                 int64_t C, int64_t D, int32_t block, int8_t* Y, float* SY, float* Y_f32, void* ws,
                                 size_t ws_bytes, void* stream) {
  using namespace jf;
  (void)ws; (void)ws_bytes;
  int32_t rc = check_linear(X, SX, W, SW, N, C, D, block);
  if (rc == JF_OK) rc = check_out(Y, SY, Y_f32, true);
  if (rc != JF_OK) return rc;
  GemmArgs g = make_args(0, X, SX, W, SW, N, C, D, block);
  g.Oq = Y; g.Os = SY; g.Of = Y_f32;
  launch_gemm(0, block, g, false, reinterpret_cast<hipStream_t>(stream));
  return launch_status();
}

extern "C" int32_t jf_linear_dgrad(const int8_t* dY, const float* SdY, const int8_t* W, const float* SW, int64_t N,
                                   int64_t C, int64_t D, int32_t block, int8_t* dX, float* SdX, float* dX_f32,
                                   void* ws, size_t ws_bytes, void* stream) {
  using namespace jf;
  (void)ws; (void)ws_bytes;
  int32_t rc = check_linear(dY, SdY, W, SW, N, C, D, block);
  if (rc == JF_OK) rc = check_out(dX, SdX, dX_f32, true);
  if (rc != JF_OK) return rc;
  GemmArgs g = make_args(1, dY, SdY, W, SW, N, C, D, block);
  g.Oq = dX; g.Os = SdX; g.Of = dX_f32;
  launch_gemm(1, block, g, false, reinterpret_cast<hipStream_t>(stream));
  return launch_status();
}

extern "C" int32_t jf_linear_wgrad(const int8_t* dY, const float* SdY, const int8_t* X, const float* SX, int64_t N,
                                   int64_t C, int64_t D, int32_t block, int8_t* dW, float* SdW, float* dW_f32,
                                   void* ws, size_t ws_bytes, void* stream) {
  using namespace jf;
  (void)ws; (void)ws_bytes;
  int32_t rc = check_linear(dY, SdY, X, SX, N, C, D, block);
  if (rc == JF_OK) rc = check_out(dW, SdW, dW_f32, false);
  if (rc != JF_OK) return rc;
  GemmArgs g = make_args(2, dY, SdY, X, SX, N, C, D, block);
  g.Oq = dW; g.Os = SdW; g.Of = dW_f32;
  launch_gemm(2, block, g, false, reinterpret_cast<hipStream_t>(stream));
  return launch_status();
}

extern "C" int32_t jf_debug_linear_partials(int32_t which, const int8_t* A, const int8_t* Bm, int64_t N, int64_t C,
                                            int64_t D, int32_t block, int64_t kb, int32_t* out, void* stream) {
  using namespace jf;
  if (!A || !Bm || !out) return JF_ERR_NULL;
  if (which < 0 || which > 2) return JF_ERR_SHAPE;
  if (!valid_block(block)) return JF_ERR_BLOCK;
  if (!valid_dim(N, block) || !valid_dim(C, block) || !valid_dim(D, block)) return JF_ERR_SHAPE;
  if (!aligned16(A) || !aligned16(Bm) || !aligned16(out)) return JF_ERR_ALIGN;
  const int64_t K = which == 0 ? C : (which == 1 ? D : N);
  if (kb < 0 || kb >= K / block) return JF_ERR_SHAPE;
  GemmArgs g = make_args(which, A, nullptr, Bm, nullptr, N, C, D, block);
  g.dump = out;
  g.dump_kb = (int)kb;
  launch_gemm(which, block, g, true, reinterpret_cast<hipStream_t>(stream));
  return launch_status();
}
