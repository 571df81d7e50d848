// Micro-benchmark behind the choice of the Eq. 1 rounding sequence: issue cost, per element and SIMD, of
//   (a) one FP32 FMA that adds 1.5 * 2^23 (rounds x * fl32(1/s): exact ties and near-ties go either way),
//   (b) FP32 FMA + add (snaps to a 2^-15 grid first: exact ties go to even, near-ties are misjudged),
//   (c) v_cvt_f64_f32 + v_fma_f64 + v_add_f64 (rounds the exact quotient: what the library uses),
// and of the other instructions the memory-bound kernels are made of.  No memory traffic; 2-8 waves per SIMD.
#include <hip/hip_runtime.h>
#include <cstdio>
#define REP16(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15)
#define CHECK(e) do { hipError_t err_ = (e); if (err_ != hipSuccess) { printf("HIP error %d at line %d\n", (int)err_, __LINE__); return; } } while (0)

template <int MODE>
__global__ void __launch_bounds__(256) k(int iters, int* out, int seed) {
  float y[16], t[16];
  double d[16], e[16];
  for (int r = 0; r < 16; ++r) { y[r] = r + seed + threadIdx.x * 0.001f; t[r] = 0; d[r] = 0; e[r] = 0; }
  float inv = 1.0f / (1.0f + seed), M = 12582528.0f, c384 = 384.0f;
  double inv64 = 1.0 / (1.0 + seed), M1 = 1572864.0, M2 = 6755399441055744.0 - 1572864.0;
  for (int i = 0; i < iters; ++i) {
    if (MODE == 0) {
#define X(r) asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(t[r]) : "v"(y[r]), "v"(inv), "v"(M));
      REP16(X)
#undef X
    } else if (MODE == 1) {
#define X(r) asm volatile("v_fma_f32 %0, %1, %2, %3\n\tv_add_f32 %0, %0, %4" : "=&v"(t[r]) : "v"(y[r]), "v"(inv), "v"(c384), "v"(M));
      REP16(X)
#undef X
    } else if (MODE == 2) {
#define X(r) asm volatile("v_cvt_f64_f32 %0, %1\n\tv_fma_f64 %0, %0, %2, %3\n\tv_add_f64 %0, %0, %4" : "=&v"(d[r]) : "v"(y[r]), "v"(inv64), "v"(M1), "v"(M2));
      REP16(X)
#undef X
    } else if (MODE == 3) {
#define X(r) asm volatile("v_cvt_f64_f32 %0, %1" : "=v"(d[r]) : "v"(y[r]));
      REP16(X)
#undef X
    } else if (MODE == 4) {
#define X(r) asm volatile("v_fma_f64 %0, %1, %2, %3" : "=v"(d[r]) : "v"(e[r]), "v"(inv64), "v"(M1));
      REP16(X)
#undef X
    } else if (MODE == 5) {
#define X(r) asm volatile("v_add_f64 %0, %1, %2" : "=v"(d[r]) : "v"(e[r]), "v"(M2));
      REP16(X)
#undef X
    } else if (MODE == 6) {
#define X(r) asm volatile("v_cvt_f32_ubyte0 %0, %1" : "=v"(t[r]) : "v"(y[r]));
      REP16(X)
#undef X
    } else if (MODE == 7) {
#define X(r) asm volatile("v_perm_b32 %0, %1, %2, %3" : "=v"(t[r]) : "v"(y[r]), "v"(inv), "v"(M));
      REP16(X)
#undef X
    } else if (MODE == 8) {
#define X(r) asm volatile("v_max3_f32 %0, |%1|, |%2|, %0" : "+v"(t[r]) : "v"(y[r]), "v"(inv));
      REP16(X)
#undef X
    } else if (MODE == 9) {
#define X(r) asm volatile("v_exp_f32 %0, %1" : "=v"(t[r]) : "v"(y[r]));
      REP16(X)
#undef X
    } else if (MODE == 10) {
#define X(r) asm volatile("v_bfe_u32 %0, %1, 8, 8" : "=v"(t[r]) : "v"(y[r]));
      REP16(X)
#undef X
    } else if (MODE == 11) {
#define X(r) asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(t[r]) : "v"(y[r]));
      REP16(X)
#undef X
    } else if (MODE == 12) {
#define X(r) asm volatile("v_dot4_i32_i8 %0, %1, %2, %0" : "+v"(t[r]) : "v"(y[r]), "v"(inv));
      REP16(X)
#undef X
    }
  }
  float sum = 0;
  for (int r = 0; r < 16; ++r) sum += t[r] + y[r] + (float)d[r] + (float)e[r];
  if (sum == 1.2345f) out[0] = (int)sum;
}

template <int MODE>
void run(const char* name, int nops) {
  int* out;
  CHECK(hipMalloc(&out, 4));
  const int iters = 20000;
  for (int wps = 2; wps <= 8; wps += 2) {  // waves per SIMD: a workgroup of 256 threads puts one wave on each SIMD of a compute unit
    dim3 grid(256 * wps), block(256);
    hipEvent_t a, b;
    CHECK(hipEventCreate(&a));
    CHECK(hipEventCreate(&b));
    k<MODE><<<grid, block>>>(100, out, 1);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(a));
    k<MODE><<<grid, block>>>(iters, out, 1);
    CHECK(hipEventRecord(b));
    CHECK(hipEventSynchronize(b));
    float ms;
    CHECK(hipEventElapsedTime(&ms, a, b));
    const double ns = ms * 1e6 / iters / wps;  // per wave-iteration (16 elements per lane) on a SIMD
    printf("%-34s w/SIMD %d: %7.1f ns per 16 elements = %6.1f cyc@2.4GHz | per element %5.2f cyc | per instruction %5.2f cyc\n", name, wps,
           ns, ns * 2.4, ns * 2.4 / 16, ns * 2.4 / nops);
    CHECK(hipEventDestroy(a));
    CHECK(hipEventDestroy(b));
  }
  CHECK(hipFree(out));
}

int main() {
  run<0>("fma32 (x * fl32(1/s))", 16);
  run<1>("fma32 + add32 (snap, round)", 32);
  run<2>("cvt64 + fma64 + add64 (exact)", 48);
  run<3>("v_cvt_f64_f32", 16);
  run<4>("v_fma_f64", 16);
  run<5>("v_add_f64", 16);
  run<6>("v_cvt_f32_ubyte0", 16);
  run<7>("v_perm_b32", 16);
  run<8>("v_max3_f32 with |.|", 16);
  run<9>("v_exp_f32", 16);
  run<10>("v_bfe_u32", 16);
  run<11>("v_cvt_f32_i32", 16);
  run<12>("v_dot4_i32_i8", 16);
  return 0;
}
