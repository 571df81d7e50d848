// gemm_kernel instances of the wgrad product at block size 128 (a translation unit of its own for build time).
#include "jf_gemm_kernel.hpp"

JF_GEMM_INSTANCE(launch_gemm_wgrad_b128, 128, false, false)
