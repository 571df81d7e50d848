// Micro-benchmark of the GEMM's inner pattern with true data dependences and no memory traffic: two INT32 tiles in
// ordinary VGPRs (as in the GEMM kernel) rotate; per unit a chain of B/32 MFMAs runs into one tile while the other,
// which the previous chain wrote, is folded (16 cvt + 16 fmac, Sec. 5.3), a share of the fold after every MFMA.
// The rates it prints are the ceilings the GEMM's K loop is compared with.
#include <hip/hip_runtime.h>
#include <cstdio>
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

template <int NC>
__global__ void __launch_bounds__(256) k(int iters, int* out, int seed) {
  v4i a = {seed + (int)threadIdx.x, seed * 3, seed * 5, seed * 7}, b = {seed * 11, seed * 13, (int)threadIdx.x, seed};
  v16i T0 = {0}, T1 = {0};
  float acc[16];
  for (int r = 0; r < 16; ++r) acc[r] = 0.f;
  float t = 1.0f + seed;
#define MFMA0(dst) asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, 0" : "=v"(dst) : "v"(a), "v"(b))
#define MFMAC(dst) asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+v"(dst) : "v"(a), "v"(b))
#define FOLD(src, R0, R1)                                                                      \
  _Pragma("unroll") for (int r = R0; r < R1; ++r) {                                            \
    float c;                                                                                   \
    asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(c) : "v"(src[r]));                              \
    asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[r]) : "v"(t), "v"(c));                     \
  }
  for (int it = 0; it < iters; ++it) {
    if (NC == 1) {
      MFMA0(T0); FOLD(T1, 0, 16)
      MFMA0(T1); FOLD(T0, 0, 16)
    } else if (NC == 2) {
      MFMA0(T0); FOLD(T1, 0, 8) MFMAC(T0); FOLD(T1, 8, 16)
      MFMA0(T1); FOLD(T0, 0, 8) MFMAC(T1); FOLD(T0, 8, 16)
    } else {
      MFMA0(T0); FOLD(T1, 0, 4) MFMAC(T0); FOLD(T1, 4, 8) MFMAC(T0); FOLD(T1, 8, 12) MFMAC(T0); FOLD(T1, 12, 16)
      MFMA0(T1); FOLD(T0, 0, 4) MFMAC(T1); FOLD(T0, 4, 8) MFMAC(T1); FOLD(T0, 8, 12) MFMAC(T1); FOLD(T0, 12, 16)
    }
  }
  float s = 0;
  for (int r = 0; r < 16; ++r) s += acc[r] + T0[r] + T1[r];
  if (s == 1.2345f) out[0] = (int)s;
}

template <int NC>
void run(int wps) {
  int* out; (void)hipMalloc(&out, 4);
  const int iters = 20000;
  hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  k<NC><<<256 * wps, 256>>>(100, out, 1);
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0);
  k<NC><<<256 * wps, 256>>>(iters, out, 1);
  (void)hipEventRecord(e1);
  (void)hipDeviceSynchronize();
  float ms; (void)hipEventElapsedTime(&ms, e0, e1);
  double ns = ms * 1e6 / iters / wps / (2 * NC);
  printf("block %3d (chain of %d), tiles in VGPRs, %d waves/SIMD: %6.1f ns per MFMA -> %6.0f TOP/s\n", 32 * NC, NC, wps, ns,
         65536.0 * 1024 / (ns * 1e-9) * 1e-12);
  (void)hipFree(out);
}

int main() {
  for (int w : {2, 3, 4}) { run<1>(w); run<2>(w); run<4>(w); }
  return 0;
}
