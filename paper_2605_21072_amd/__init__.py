"""MI355X-native dual-scale W8A8 linear layer of Q-ARVD: thin Python binding over libqarvd.so.

The three operations live in hand-written HIP kernels behind a C ABI (``include/qarvd.h``); this
package only marshals arguments.  PyTorch supplies device memory and streams, nothing else.
"""
from .binding import (  # noqa: F401
    ACT_GELU_TANH,
    ACT_NONE,
    DualScaleWeight,
    QarvdError,
    gemm_num_variants,
    gemm_variant_name,
    lib_path,
    load_library,
    packed_channel_map,
    packed_k,
    packed_ld,
    packed_normal_offset,
    probe_mfma_peak,
    q8_gemm_num_variants,
    quant_act,
    quant_act_static,
    quantize_weight,
    quantize_weight_static,
    quantize_weight_static_max_k,
    quantize_weight_workspace,
    w8a8_dual_gemm,
    w8a8_dual_gemm_q8,
    w8a8_linear,
)
