"""MI355X-native hot path of AAAC: activation importance, weighted Lloyd
iterations learning two 16-entry codebooks, 4-bit encode and dequant, as HIP
kernels for gfx950 behind a C ABI (include/aaac.h).

The functions re-exported here only marshal arguments into that library; they
raise if it has not been built.
"""
from .binding import (  # noqa: F401
    AaacError, aaac_act_stats, aaac_act_stats_static, aaac_act_stats_workspace, aaac_dequant, aaac_dequant_sel, aaac_encode,
    aaac_encode_sel, aaac_fit, aaac_fit_batch, aaac_fit_batch_workspace, aaac_fit_nested, aaac_gemm_w4a16, aaac_gemm_w4a16_workspace, aaac_gemv_w4a16,
    aaac_fit_nested_workspace, aaac_fit_workspace, aaac_quantile_init, aaac_quantile_init_workspace, library, library_path, make_layers, sel_stride,
    NVFP4, INT4,
)
