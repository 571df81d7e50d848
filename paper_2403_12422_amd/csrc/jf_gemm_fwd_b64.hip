// gemm_kernel instances of the fwd product at block size 64 (a translation unit of its own for build time).
#include "jf_gemm_kernel.hpp"

JF_GEMM_INSTANCE(launch_gemm_fwd_b64, 64, true, true)
