"""MI355X-native layer-wise Hessian-aware quantization (hot path of the paper's layer-wise PTQ stage).

The computation lives in libonecomp.so (hand-written HIP for gfx950, C ABI in include/onecomp.h);
this package is the thin Python binding around it plus the seeded synthetic-input generator.
"""
from .binding import (  # noqa: F401
    EXPORTED_SYMBOLS,
    LIB_PATH,
    OnecompError,
    load_library,
    onecomp_accumulate_describe,
    onecomp_accumulate_workspace_bytes,
    onecomp_crossgram_accumulate,
    onecomp_factor_workspace_bytes,
    onecomp_hessian_accumulate,
    onecomp_hessian_factor,
    onecomp_jointq_refine,
    onecomp_jointq_workspace_bytes,
    onecomp_mfma_rate_probe,
    onecomp_qep_target,
    onecomp_qep_workspace_bytes,
    onecomp_quantize_layer,
    onecomp_quantize_workspace_bytes,
    onecomp_rtn_sensitivity,
    onecomp_rtn_sensitivity_static,
    onecomp_version,
    status_string,
)
