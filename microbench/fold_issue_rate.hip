// Micro-benchmark behind the ceilings quoted for the per-block INT8 GEMM: issue rate of the vector instructions of
// the dequantize fold of Sec. 5.3 (one int->float conversion and one FMA per output element and K-block), alone
// and next to v_mfma_i32_32x32x32_i8, at 2-4 resident waves per SIMD.  No memory traffic.  The three mixes
// "1 mfma + 32 / 16 / 8 vector instructions" are the inner loops of quantization block sizes 32 / 64 / 128.
#include <hip/hip_runtime.h>
#include <cstdio>
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

#define REP16(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15)

template <int MODE>
__global__ void __launch_bounds__(256) k(int iters, int* out, int seed) {
  v4i a = {seed + (int)threadIdx.x, seed * 3, seed * 5, seed * 7}, b = {seed * 11, seed * 13, (int)threadIdx.x, seed};
  v16i c0, c1;
  float acc[16], tmp[16];
  for (int r = 0; r < 16; ++r) { acc[r] = 0.f; tmp[r] = r; c0[r] = seed * r; c1[r] = seed + r; }
  float t = 1.0f + seed, M = 12582912.0f;
  for (int i = 0; i < iters; ++i) {
    if (MODE == 0) {         // 16 v_cvt_f32_i32
#define X(r) asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(tmp[r]) : "v"(c0[r]));
      REP16(X)
#undef X
    } else if (MODE == 1) {  // 16 v_fmac_f32
#define X(r) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[r]) : "v"(t), "v"(tmp[r]));
      REP16(X)
#undef X
    } else if (MODE == 2) {  // 16 v_sub_f32
#define X(r) asm volatile("v_sub_f32 %0, %1, %2" : "=v"(tmp[r]) : "v"(c0[r]), "v"(M));
      REP16(X)
#undef X
    } else if (MODE == 3) {  // 16 cvt + 16 fmac interleaved by 4
#define X(r) asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(tmp[r]) : "v"(c0[r]));
#define Y(r) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[r]) : "v"(t), "v"(tmp[r]));
      X(0) X(1) X(2) X(3) Y(0) Y(1) Y(2) Y(3) X(4) X(5) X(6) X(7) Y(4) Y(5) Y(6) Y(7)
      X(8) X(9) X(10) X(11) Y(8) Y(9) Y(10) Y(11) X(12) X(13) X(14) X(15) Y(12) Y(13) Y(14) Y(15)
#undef X
#undef Y
    } else if (MODE == 4) {  // 16 sub + 16 fmac
#define X(r) asm volatile("v_sub_f32 %0, %1, %2" : "=v"(tmp[r]) : "v"(c0[r]), "v"(M));
#define Y(r) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[r]) : "v"(t), "v"(tmp[r]));
      X(0) X(1) X(2) X(3) Y(0) Y(1) Y(2) Y(3) X(4) X(5) X(6) X(7) Y(4) Y(5) Y(6) Y(7)
      X(8) X(9) X(10) X(11) Y(8) Y(9) Y(10) Y(11) X(12) X(13) X(14) X(15) Y(12) Y(13) Y(14) Y(15)
#undef X
#undef Y
    } else if (MODE == 5) {  // mfma (independent of the VALU work) + 16 cvt + 16 fmac
      c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
#define X(r) asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(tmp[r]) : "v"(c0[r]));
#define Y(r) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[r]) : "v"(t), "v"(tmp[r]));
      X(0) X(1) X(2) X(3) Y(0) Y(1) Y(2) Y(3) X(4) X(5) X(6) X(7) Y(4) Y(5) Y(6) Y(7)
      X(8) X(9) X(10) X(11) Y(8) Y(9) Y(10) Y(11) X(12) X(13) X(14) X(15) Y(12) Y(13) Y(14) Y(15)
#undef X
#undef Y
    } else if (MODE == 6) {  // mfma + 16 fmac only
      c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
#define Y(r) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[r]) : "v"(t), "v"(tmp[r]));
      REP16(Y)
#undef Y
    } else if (MODE == 7) {  // mfma + 8 VALU (4 cvt + 4 fmac): the B = 128 mix
      c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
#define X(r) asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(tmp[r]) : "v"(c0[r]));
#define Y(r) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[r]) : "v"(t), "v"(tmp[r]));
      X(0) X(1) X(2) X(3) Y(0) Y(1) Y(2) Y(3)
#undef X
#undef Y
    } else if (MODE == 8) {  // mfma + 16 VALU: the B = 64 mix
      c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
#define X(r) asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(tmp[r]) : "v"(c0[r]));
#define Y(r) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[r]) : "v"(t), "v"(tmp[r]));
      X(0) X(1) X(2) X(3) Y(0) Y(1) Y(2) Y(3) X(4) X(5) X(6) X(7) Y(4) Y(5) Y(6) Y(7)
#undef X
#undef Y
    } else if (MODE == 9) {  // mfma only (one chain)
      c1 = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c1, 0, 0, 0);
    }
  }
  float s = 0;
  for (int r = 0; r < 16; ++r) s += acc[r] + tmp[r] + c1[r];
  if (s == 1.2345f) out[0] = (int)s;
}

template <int MODE>
void run(const char* name, int wps, int nvalu, int nmfma) {
  int* out;
  (void)hipMalloc(&out, 4);
  const int iters = 40000;
  dim3 grid(256 * wps), block(256);
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  k<MODE><<<grid, block>>>(100, out, 1);
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0);
  k<MODE><<<grid, block>>>(iters, out, 1);
  (void)hipEventRecord(e1);
  (void)hipDeviceSynchronize();
  float ms; (void)hipEventElapsedTime(&ms, e0, e1);
  double ns_per_iter_simd = ms * 1e6 / iters / wps;   // SIMD time per wave-iteration
  printf("%-34s w/SIMD %d: %7.1f ns per wave-iter on a SIMD = %6.1f cyc@2.4GHz | per VALU %5.2f cyc | MFMA rate %6.1f TOP/s\n", name, wps,
         ns_per_iter_simd, ns_per_iter_simd * 2.4, nvalu ? ns_per_iter_simd * 2.4 / nvalu : 0.0,
         nmfma * 65536.0 * 1024 / (ns_per_iter_simd * 1e-9) * 1e-12);
  (void)hipFree(out);
}

int main() {
  for (int w : {2, 3, 4}) {
    run<0>("16 cvt_f32_i32", w, 16, 0);
    run<1>("16 fmac_f32", w, 16, 0);
    run<2>("16 sub_f32", w, 16, 0);
    run<3>("16 cvt + 16 fmac", w, 32, 0);
    run<4>("16 sub + 16 fmac", w, 32, 0);
    run<9>("1 mfma", w, 0, 1);
    run<5>("1 mfma + 16 cvt + 16 fmac", w, 32, 1);
    run<6>("1 mfma + 16 fmac", w, 16, 1);
    run<8>("1 mfma + 8 cvt + 8 fmac", w, 16, 1);
    run<7>("1 mfma + 4 cvt + 4 fmac", w, 8, 1);
  }
  return 0;
}
