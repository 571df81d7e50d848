// gemm_pair_kernel instances: input gradient and weight gradient of a block-32 layer in one launch (a translation
// unit of its own for build time).
#define JF_GEMM_PAIR_INSTANCES
#include "jf_gemm_kernel.hpp"

namespace jf {
bool launch_gemm_bwd_pair_b32(const GemmArgs& dgrad, const GemmArgs& wgrad, hipStream_t st) {
  return launch_bwd_pair_b32(dgrad, wgrad, st);
}
}  // namespace jf
