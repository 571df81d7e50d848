// A model of the GEMM's K loop per tile shape and block size, written the naive way: per unit (one 32x32 sub-block x
// one quantization block) a chain of NC = B/32 MFMAs with the fold of the previous unit's INT32 tile woven in
// (Sec. 5.3), READS ds_read_b128 per MFMA issued right before it, and per stage LOADS direct-to-LDS loads per wave
// (scalar-base form), the wait for the stage after next, a workgroup barrier and the scalar scale loads.  "bare fold"
// leaves out everything but the MFMAs and the fold.  It shows what a loop with this instruction mix costs on the
// chip, shape against shape; the real kernel reads its fragments earlier and does a little better than the model.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

template <int NC, int WAVES, int LOADS, int UNITS, int WPS, bool FULL, int READS = 1>
__global__ void __launch_bounds__(64 * WAVES, WPS) k(int iters, int* out, int seed, const int8_t* src, const float* scales) {
  constexpr int STAGE = LOADS * WAVES * 1024;
  __shared__ __align__(1024) int8_t ring[3][STAGE];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v4i a = {seed + (int)threadIdx.x, seed * 3, seed * 5, seed * 7}, b = {seed * 11, seed * 13, (int)threadIdx.x, seed};
  v16i T0 = {0}, T1 = {0};
  float acc[4][16];
  for (int q = 0; q < 4; ++q) for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;
  for (int i = threadIdx.x; i < 3 * STAGE / 4; i += 64 * WAVES) ((int*)ring)[i] = i * seed;
  __syncthreads();
  const uint32_t loff = (wave * 64 + lane) * 16;
  typedef const __attribute__((address_space(4))) float* cptr;
  cptr sc = (cptr)scales;
#define MFMA0(dst, A, Bv) asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, 0" : "=v"(dst) : "v"(A), "v"(Bv))
#define MFMAC(dst, A, Bv) asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+v"(dst) : "v"(A), "v"(Bv))
#define FOLDP(src, Q, tt, R0, R1)                                                              \
  _Pragma("unroll") for (int r = R0; r < R1; ++r) {                                            \
    float c;                                                                                   \
    asm volatile("v_cvt_f32_i32 %0, %1" : "=v"(c) : "v"(src[r]));                              \
    asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(acc[Q][r]) : "v"(tt), "v"(c));                 \
  }
  for (int it = 0; it < iters; ++it) {
    const int slot = it % 3;
    float s0 = 1.0f, s1 = 1.0f;
    if (FULL) { s0 = sc[(it & 63)]; s1 = sc[64 + (it & 63)]; }
    const float tt = s0 * s1 + seed;
#pragma unroll
    for (int u = 0; u < UNITS; ++u) {
#pragma unroll
      for (int j = 0; j < NC; ++j) {
        v4i f = a;
        v4i f2 = b;
        if (FULL) f = *reinterpret_cast<const v4i*>(&ring[slot][(((u * NC + j) * 64 + lane) * 16) % STAGE]);
        if (FULL && READS == 2) f2 = *reinterpret_cast<const v4i*>(&ring[slot][(((u * NC + j) * 64 + lane) * 16 + STAGE / 2) % STAGE]);
        if (u & 1) {
          if (j == 0) MFMA0(T1, f, f2); else MFMAC(T1, f, f2);
          FOLDP(T0, (u & 3), tt, 16 * j / NC, 16 * (j + 1) / NC)
        } else {
          if (j == 0) MFMA0(T0, f, f2); else MFMAC(T0, f, f2);
          FOLDP(T1, (u & 3), tt, 16 * j / NC, 16 * (j + 1) / NC)
        }
      }
    }
    if (FULL) {
      const int ns = (it + 2) % 3;
#pragma unroll
      for (int i = 0; i < LOADS; ++i) {
        const int8_t* ub = src + (size_t)blockIdx.x * 65536 + ((it * LOADS + i) & 3) * (WAVES * 1024);
        const uint32_t la = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)&ring[ns][(i * WAVES + wave) * 1024]);
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(loff), "s"(ub), "s"(la) : "memory", "m0");
      }
      __builtin_amdgcn_s_waitcnt((LOADS & 15) | (7 << 4) | (15 << 8));
      asm volatile("s_barrier" ::: "memory");
    }
  }
  if (FULL) __builtin_amdgcn_s_waitcnt((7 << 4) | (15 << 8));
  float s = 0;
  for (int q = 0; q < 4; ++q) for (int r = 0; r < 16; ++r) s += acc[q][r];
  for (int r = 0; r < 16; ++r) s += T0[r] + T1[r];
  if (s == 1.2345f) out[0] = (int)s;
}

template <int NC, int WAVES, int LOADS, int UNITS, int WPS, bool FULL, int READS = 1>
void run(const char* name, const int8_t* src, const float* scales) {
  int* out; (void)hipMalloc(&out, 4);
  const int iters = 2000;
  const int wgs = 256 * (WPS * 4 / WAVES);
  hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  k<NC, WAVES, LOADS, UNITS, WPS, FULL, READS><<<wgs, 64 * WAVES>>>(50, out, 1, src, scales);
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0);
  k<NC, WAVES, LOADS, UNITS, WPS, FULL, READS><<<wgs, 64 * WAVES>>>(iters, out, 1, src, scales);
  (void)hipEventRecord(e1);
  (void)hipDeviceSynchronize();
  float ms; (void)hipEventElapsedTime(&ms, e0, e1);
  double ns = ms * 1e6 / iters / WPS / (UNITS * NC);
  printf("%-44s %s %d waves/SIMD: %6.1f ns per MFMA -> %6.0f TOP/s\n", name, FULL ? "full loop" : "bare fold", WPS, ns,
         65536.0 * 1024 / (ns * 1e-9) * 1e-12);
  fflush(stdout);
  (void)hipFree(out);
}

int main() {
  int8_t* src; float* scales;
  (void)hipMalloc(&src, (size_t)1024 * 65536 + 65536);
  (void)hipMemset(src, 1, (size_t)1024 * 65536 + 65536);
  (void)hipMalloc(&scales, 4096);
  (void)hipMemset(scales, 0, 4096);
  // block 32: 128x128 tile, 4 waves, stage of 64 K bytes: 4 loads per wave, 8 units per wave and stage, 3 workgroups per CU
  run<1, 4, 4, 8, 3, false>("B=32  128x128, 4 waves", src, scales);
  run<1, 4, 4, 8, 3, true>("B=32  128x128, 4 waves", src, scales);
  // block 32, 64x64 tile: 4 waves of one sub-block, stage of 64 K bytes: 2 loads per wave, 2 units, 2 fragment reads per unit
  run<1, 4, 2, 2, 3, true, 2>("B=32  64x64, 4 waves, KC 64", src, scales);
  run<1, 4, 4, 4, 3, true, 2>("B=32  64x64, 4 waves, KC 128", src, scales);
  run<1, 4, 2, 2, 4, true, 2>("B=32  64x64, 4 waves, KC 64", src, scales);
  // a 64x64 tile whose four waves split K (each wave 2x2 sub-blocks of one K step per stage of 128 K bytes: 4 loads,
  // 4 units, one fragment read per unit); not built -- it would sum every output element in four chains
  run<1, 4, 4, 4, 3, true, 1>("B=32  64x64, 4 waves splitting K, KC 128", src, scales);
  // block 64: same tile, a stage holds one quantization block: 4 units of 2 MFMAs
  run<2, 4, 4, 4, 3, false>("B=64  128x128, 4 waves", src, scales);
  run<2, 4, 4, 4, 3, true>("B=64  128x128, 4 waves", src, scales);
  // block 128: 256x128 tile, 8 waves, stage of 128 K bytes: 6 loads per wave, 4 units of 4 MFMAs, 1 workgroup per CU
  run<4, 8, 6, 4, 2, false>("B=128 256x128, 8 waves", src, scales);
  run<4, 8, 6, 4, 2, true>("B=128 256x128, 8 waves", src, scales);
  return 0;
}
