// Micro-benchmark of what the GEMM's K loop costs on top of the bare fold (block size 32): the B = 32 pattern of
// fold_chain_rate (one MFMA + 16 cvt + 16 fmac per unit, two INT32 tiles rotating) with the other instructions of
// the real loop added one kind at a time:
//   0 nothing;  1 + one ds_read_b128 per unit feeding the MFMAs;  2 + a workgroup barrier every 8 units;
//   3 + four direct-to-LDS loads per 8 units and wave (64-bit per-lane addresses) into a ring of three 16 KB stages;
//   4 + scalar loads and the product of two block scales per pair of units;
//   5 = 4 with the loads in the scalar-base + 32-bit-lane-offset form (no vector ALU on addresses);
//   6 = 5 with the eight fragment reads of a stage issued at once instead of two by two.
// Three workgroups of four waves per compute unit (three waves per SIMD), as the 128x128 tile runs.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef const __attribute__((address_space(1))) void* gbl_ptr;

template <int V>
__global__ void __launch_bounds__(256, 3) k(int iters, int* out, int seed, const int8_t* src, const float* scales) {
  __shared__ __align__(1024) int8_t ring[3][16384];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v4i a = {seed + (int)threadIdx.x, seed * 3, seed * 5, seed * 7}, b = {seed * 11, seed * 13, (int)threadIdx.x, seed};
  v16i T0 = {0}, T1 = {0};
  float acc[4][16];
  for (int q = 0; q < 4; ++q) for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;
  float t = 1.0f + seed;
  for (int i = threadIdx.x; i < 3 * 16384 / 4; i += 256) ((int*)ring)[i] = i * seed;
  __syncthreads();
  const int8_t* gsrc = src + (size_t)blockIdx.x * 65536 + (wave * 64 + lane) * 16;
  const uint32_t loff = (wave * 64 + lane) * 16;
  typedef const __attribute__((address_space(4))) float* cptr;
  cptr sc = (cptr)scales;
#define MFMA0(dst, A, Bv) asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, 0" : "=v"(dst) : "v"(A), "v"(Bv))
#define FOLD(src, Q, tt)                                                                       \
  _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                             \
    float c;                                                                                   \
    asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(c) : "v"(src[r]));                              \
    asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[Q][r]) : "v"(tt), "v"(c));                 \
  }
  for (int it = 0; it < iters; ++it) {
    const int slot = it % 3;
    float s0 = t, s1 = t;
    if (V >= 4) { s0 = sc[(it & 63)]; s1 = sc[64 + (it & 63)]; }
    if (V >= 6) {
      // all eight fragments of the stage are read at once, ahead of their use (as the GEMM kernel does)
      v4i f[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) f[u] = *reinterpret_cast<const v4i*>(&ring[slot][(u & 1) * 8192 + (u * 64 + lane) * 16]);
      const float tt = s0 * s1;
#pragma unroll
      for (int u = 0; u < 8; u += 2) {
        MFMA0(T0, f[u], b); FOLD(T1, (u & 3), tt)
        MFMA0(T1, a, f[u + 1]); FOLD(T0, ((u + 1) & 3), tt)
      }
    } else {
#pragma unroll
    for (int u = 0; u < 8; u += 2) {
      v4i fa = a, fb = b;
      if (V >= 1) {
        fa = *reinterpret_cast<const v4i*>(&ring[slot][(u * 64 + lane) * 16]);
        fb = *reinterpret_cast<const v4i*>(&ring[slot][8192 + ((u + 1) * 64 + lane) * 16]);
      }
      float tt = t;
      if (V >= 4) tt = s0 * s1;
      MFMA0(T0, fa, b); FOLD(T1, (u & 3), tt)
      MFMA0(T1, a, fb); FOLD(T0, ((u + 1) & 3), tt)
    }
    }
    if (V >= 3) {
      const int ns = (it + 2) % 3;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (V >= 5) {
          const int8_t* ub = src + (size_t)blockIdx.x * 65536 + ((it * 4 + i) & 15) * 4096;   // uniform
          const uint32_t la = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)&ring[ns][(i * 4 + wave) * 1024]);
          asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(loff), "s"(ub), "s"(la) : "memory", "m0");
        } else
        __builtin_amdgcn_global_load_lds((gbl_ptr)(gsrc + ((it * 4 + i) & 15) * 4096), (lds_ptr)(&ring[ns][(i * 4 + wave) * 1024]), 16, 0, 0);
      __builtin_amdgcn_s_waitcnt((4 & 15) | (7 << 4) | (15 << 8));   // vmcnt(4): the previous stage has landed
    }
    if (V >= 2) asm volatile("s_barrier" ::: "memory");
  }
  if (V >= 3) __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));
  float s = 0;
  for (int q = 0; q < 4; ++q) for (int r = 0; r < 16; ++r) s += acc[q][r];
  for (int r = 0; r < 16; ++r) s += T0[r] + T1[r];
  if (s == 1.2345f) out[0] = (int)s;
}

template <int V>
void run(int wgs_per_cu, const int8_t* src, const float* scales) {
  int* out; (void)hipMalloc(&out, 4);
  const int iters = 4000;
  hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  k<V><<<256 * wgs_per_cu, 256>>>(50, out, 1, src, scales);
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0);
  k<V><<<256 * wgs_per_cu, 256>>>(iters, out, 1, src, scales);
  (void)hipEventRecord(e1);
  (void)hipDeviceSynchronize();
  float ms; (void)hipEventElapsedTime(&ms, e0, e1);
  double ns = ms * 1e6 / iters / wgs_per_cu / 8;
  printf("variant %d, %d waves/SIMD: %6.1f ns per MFMA+fold -> %6.0f TOP/s\n", V, wgs_per_cu, ns, 65536.0 * 1024 / (ns * 1e-9) * 1e-12);
  fflush(stdout);
  (void)hipFree(out);
}

int main() {
  int8_t* src; float* scales;
  (void)hipMalloc(&src, (size_t)256 * 3 * 65536 + 65536);
  (void)hipMemset(src, 1, (size_t)256 * 3 * 65536 + 65536);
  (void)hipMalloc(&scales, 4096);
  (void)hipMemset(scales, 0, 4096);
  for (int w : {2, 3}) { run<0>(w, src, scales); run<1>(w, src, scales); run<2>(w, src, scales); run<3>(w, src, scales); run<4>(w, src, scales); run<5>(w, src, scales); run<6>(w, src, scales); }
  return 0;
}
