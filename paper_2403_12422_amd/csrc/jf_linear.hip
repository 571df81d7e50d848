// Per-block INT8 linear layer (Sec. 5, Alg. 1): C entry points of forward, dgrad, wgrad and the INT32-partial
// test hook.  The kernel lives in jf_gemm_kernel.hpp and is instantiated per product and block size in
// jf_gemm_<product>_b<block>.hip.
#include "jf_gemm_kernel.hpp"

namespace jf {

void launch_gemm_fwd_b32(const GemmArgs& a, bool dump, hipStream_t st);
void launch_gemm_fwd_b64(const GemmArgs& a, bool dump, hipStream_t st);
void launch_gemm_fwd_b128(const GemmArgs& a, bool dump, hipStream_t st);
void launch_gemm_dgrad_b32(const GemmArgs& a, bool dump, hipStream_t st);
void launch_gemm_dgrad_b64(const GemmArgs& a, bool dump, hipStream_t st);
void launch_gemm_dgrad_b128(const GemmArgs& a, bool dump, hipStream_t st);
void launch_gemm_wgrad_b32(const GemmArgs& a, bool dump, hipStream_t st);
void launch_gemm_wgrad_b64(const GemmArgs& a, bool dump, hipStream_t st);
void launch_gemm_wgrad_b128(const GemmArgs& a, bool dump, hipStream_t st);
bool launch_gemm_bwd_pair_b32(const GemmArgs& dgrad, const GemmArgs& wgrad, hipStream_t st);

std::atomic<int> g_forced_shape{0};

// which: 0 forward, 1 dgrad, 2 wgrad
static void launch_gemm(int which, int block, const GemmArgs& a, bool dump, hipStream_t st) {
  typedef void (*launcher)(const GemmArgs&, bool, hipStream_t);
  static const launcher table[3][3] = {
      {launch_gemm_fwd_b32, launch_gemm_fwd_b64, launch_gemm_fwd_b128},
      {launch_gemm_dgrad_b32, launch_gemm_dgrad_b64, launch_gemm_dgrad_b128},
      {launch_gemm_wgrad_b32, launch_gemm_wgrad_b64, launch_gemm_wgrad_b128},
  };
  table[which][block == 32 ? 0 : (block == 64 ? 1 : 2)](a, dump, st);
}

static int32_t check_linear(const void* p0, const void* p1, const void* p2, const void* p3, int64_t N, int64_t C,
                            int64_t D, int32_t block) {
  if (!p0 || !p1 || !p2 || !p3) return JF_ERR_NULL;
  if (!valid_block(block)) return JF_ERR_BLOCK;
  if (!valid_dim(N, block) || !valid_dim(C, block) || !valid_dim(D, block)) return JF_ERR_SHAPE;
  if (!valid_size(N, C) || !valid_size(N, D) || !valid_size(D, C)) return JF_ERR_SHAPE;
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

extern "C" int32_t jf_linear_bwd(const int8_t* dY, const float* SdY, const int8_t* W, const float* SW, const int8_t* X,
                                 const float* SX, int64_t N, int64_t C, int64_t D, int32_t block, int8_t* dX, float* SdX,
                                 float* dX_f32, int8_t* dW, float* SdW, float* dW_f32, void* ws, size_t ws_bytes,
                                 void* stream) {
  using namespace jf;
  (void)ws; (void)ws_bytes;
  int32_t rc = check_linear(dY, SdY, W, SW, N, C, D, block);
  if (rc == JF_OK) rc = check_linear(dY, SdY, X, SX, N, C, D, block);
  if (rc == JF_OK) rc = check_out(dX, SdX, dX_f32, true);
  if (rc == JF_OK) rc = check_out(dW, SdW, dW_f32, false);
  if (rc != JF_OK) return rc;
  GemmArgs gd = make_args(1, dY, SdY, W, SW, N, C, D, block);
  gd.Oq = dX; gd.Os = SdX; gd.Of = dX_f32;
  GemmArgs gw = make_args(2, dY, SdY, X, SX, N, C, D, block);
  gw.Oq = dW; gw.Os = SdW; gw.Of = dW_f32;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (block != 32 || !launch_gemm_bwd_pair_b32(gd, gw, st)) {   // shapes that fill the chip on their own: two launches
    launch_gemm(1, block, gd, false, st);
    rc = launch_status();
    if (rc != JF_OK) return rc;
    launch_gemm(2, block, gw, false, st);
  }
  return launch_status();
}

extern "C" int32_t jf_debug_linear_partials(int32_t which, const int8_t* A, const int8_t* Bm, int64_t N, int64_t C,
                                            int64_t D, int32_t block, int64_t kb, int32_t* out, void* stream) {
  using namespace jf;
  if (!A || !Bm || !out) return JF_ERR_NULL;
  if (which < 0 || which > 2) return JF_ERR_SHAPE;
  if (!valid_block(block)) return JF_ERR_BLOCK;
  if (!valid_dim(N, block) || !valid_dim(C, block) || !valid_dim(D, block)) return JF_ERR_SHAPE;
  if (!valid_size(N, C) || !valid_size(N, D) || !valid_size(D, C)) return JF_ERR_SHAPE;
  if (!aligned16(A) || !aligned16(Bm) || !aligned16(out)) return JF_ERR_ALIGN;
  const int64_t K = which == 0 ? C : (which == 1 ? D : N);
  if (kb < 0 || kb >= K / block) return JF_ERR_SHAPE;
  GemmArgs g = make_args(which, A, nullptr, Bm, nullptr, N, C, D, block);
  g.dump = out;
  g.dump_kb = (int)kb;
  launch_gemm(which, block, g, true, reinterpret_cast<hipStream_t>(stream));
  return launch_status();
}

extern "C" int32_t jf_debug_set_gemm_shape(int32_t shape) {
  if (shape != 0 && shape != 1 && shape != 4 && shape != 6 && shape != 7 && shape != 8) return JF_ERR_SHAPE;
  jf::g_forced_shape.store(shape, std::memory_order_relaxed);
  return JF_OK;
}
