// Entry points that launch nothing: error reporting and workspace sizing.
#include "jf_common.hpp"

namespace jf {
thread_local int32_t g_last_hip_error = 0;
}

extern "C" int32_t jf_last_hip_error(void) { return jf::g_last_hip_error; }

extern "C" const char* jf_error_string(int32_t code) {
  switch (code) {
    case JF_OK: return "JF_OK";
    case JF_ERR_NULL: return "JF_ERR_NULL: a required pointer is NULL";
    case JF_ERR_SHAPE: return "JF_ERR_SHAPE: dimension not positive, too large or not a multiple of block";
    case JF_ERR_BLOCK: return "JF_ERR_BLOCK: block must be 32, 64 or 128";
    case JF_ERR_ALIGN: return "JF_ERR_ALIGN: pointer or leading dimension misaligned";
    case JF_ERR_WORKSPACE: return "JF_ERR_WORKSPACE: workspace missing or too small";
    case JF_ERR_LAUNCH: return "JF_ERR_LAUNCH: a HIP call failed";
    case JF_ERR_DTYPE: return "JF_ERR_DTYPE: unknown source dtype";
    default: return "unknown jetfire error code";
  }
}

extern "C" size_t jf_workspace_bytes(int32_t op, int64_t N, int64_t C, int64_t D, int32_t block) {
  (void)D;
  if (!jf::valid_block(block) || N <= 0 || C <= 0) return 0;
  switch (op) {
    case JF_OP_LAYERNORM_BWD:
      return jf::ln_bwd_workspace_bytes(N, C);
    default:
      return 0;
  }
}
