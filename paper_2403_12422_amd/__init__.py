"""MI355X-native per-block INT8 data flow (arxiv 2403.12422): thin Python binding over libjetfire.so.

The functions in :mod:`paper_2403_12422_amd.binding` carry the names of the C ABI
(``include/jetfire.h``) and only marshal arguments; every arithmetic step runs in
the HIP kernels.  There is no CPU fallback: calling an op without the built
library or without a GPU raises.
"""
from .binding import (  # noqa: F401
    JetfireError,
    jf_add_q,
    jf_debug_linear_partials,
    jf_debug_set_gemm_shape,
    jf_dequantize_block,
    jf_dropout_q,
    jf_gelu_q,
    jf_gelu_q_bwd,
    jf_layernorm_q,
    jf_layernorm_q_bwd,
    jf_layernorm_q_bwd_static,
    jf_layernorm_q_partials,
    jf_linear_bwd,
    jf_linear_dgrad,
    jf_linear_fwd,
    jf_linear_wgrad,
    jf_quantize_block,
    jf_workspace_bytes,
    library_path,
    load_library,
)
