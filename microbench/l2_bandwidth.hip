// Micro-benchmark behind the tile-size discussion of the per-block INT8 GEMM: L2 -> compute-unit bandwidth with
// plain 16-byte global loads and with direct-to-LDS loads, for footprints inside and beyond the L2 caches.
// Each workgroup (256 threads) sweeps a private window of `win` bytes again and again; all windows together
// are `nwg * win` bytes: small totals stay in L2 (4 MB per XCD), larger ones in the 256 MB last-level cache.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdint>
typedef int v4i __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef const __attribute__((address_space(1))) void* gbl_ptr;

template <bool TO_LDS>
__global__ void __launch_bounds__(256) k(const int8_t* src, int win, int shared_by, int iters, int* out) {
  __shared__ __align__(1024) int8_t buf[65536];
  const int tid = threadIdx.x, wave = tid >> 6;
  const int8_t* base = src + (size_t)(blockIdx.x / shared_by) * win;
  v4i acc = {0, 0, 0, 0};
  for (int it = 0; it < iters; ++it) {
    for (int off = 0; off < win; off += 16384) {   // 16 KB per pass of the workgroup: 4 loads of 16 B per thread
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int8_t* p = base + off + (i * 256 + tid) * 16;
        if (TO_LDS) {
          __builtin_amdgcn_global_load_lds((gbl_ptr)p, (lds_ptr)(buf + ((off >> 14) & 3) * 16384 + 1024 * (i * 4 + wave)), 16, 0, 0);
        } else {
          v4i v = *(const v4i*)p;
          acc += v;
        }
      }
    }
    if (TO_LDS) __builtin_amdgcn_s_waitcnt(0x0070 | (15 << 8) | (0 << 14) | 8);  // vmcnt(8)
  }
  __syncthreads();
  if (TO_LDS) acc[0] = *(int*)(buf + tid * 4);
  if (acc[0] + acc[1] + acc[2] + acc[3] == 0x12345678) out[0] = 1;
}

template <bool TO_LDS>
void run(const int8_t* src, int nwg, int win, int shared_by, const char* what) {
  int* out; (void)hipMalloc(&out, 4);
  int iters = (int)(((size_t)1 << 26) / win);   // 64 MB per workgroup
  hipEvent_t e0, e1; (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  k<TO_LDS><<<nwg, 256>>>(src, win, shared_by, 2, out);
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0);
  k<TO_LDS><<<nwg, 256>>>(src, win, shared_by, iters, out);
  (void)hipEventRecord(e1);
  (void)hipDeviceSynchronize();
  float ms; (void)hipEventElapsedTime(&ms, e0, e1);
  double bytes = (double)nwg * iters * win;
  printf("%-8s %-14s wg %5d window %7d B shared by %2d (footprint %7.1f MB): %7.2f TB/s  = %5.1f B/ns per CU\n", what, TO_LDS ? "direct-to-LDS" : "to registers", nwg, win,
         shared_by, (double)(nwg / shared_by) * win / 1e6, bytes / (ms * 1e-3) * 1e-12, bytes / (ms * 1e-3) * 1e-9 / 256);
  (void)hipFree(out);
}

int main() {
  int8_t* src; (void)hipMalloc(&src, (size_t)1 << 30); (void)hipMemset(src, 1, (size_t)1 << 30);
  for (int nwg : {256, 512, 1024}) {
    for (int win : {16384, 65536, 262144}) {
      run<false>(src, nwg, win, 1, "private");
      run<true>(src, nwg, win, 1, "private");
    }
    run<false>(src, nwg, 65536, 8, "shared");
    run<true>(src, nwg, 65536, 8, "shared");
    run<true>(src, nwg, 1048576, 8, "shared");
  }
  return 0;
}
