"""MI355X-native AWEQ (arXiv 2311.01305) calibration + quantization hot path.

`paper_2311_01305_amd.binding` mirrors the C ABI of include/aweq.h one to one; every step
runs in the hand-written HIP kernels of libaweq.so.  There is no CPU fallback: calling
an op without the built library raises.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    AWEQ_F16, AWEQ_F32, AWEQ_I8, BIAS_W8A8, BIAS_WEIGHT_ONLY, AweqError, aweq_bias_correct,
    aweq_calib_stats, aweq_calib_stats_static, aweq_equalize, aweq_quant_act, aweq_quant_weight, aweq_status_string,
    aweq_w8a8_gemm, aweq_workspace_size, load_library, aweq_panel_bytes, aweq_pack_panels_i8,
    aweq_unpack_panels_i8, aweq_wonly_gemm, aweq_fold_quant_weight,
)
