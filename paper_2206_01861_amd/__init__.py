"""libzq: ZeroQuant's quantized linear layer (arXiv 2206.01861) for AMD MI355X.

Thin Python binding over the C ABI in include/zq.h.  Every step of the layer
runs in the HIP kernels of libzq.so; torch only provides device memory and the
stream.  There is no CPU fallback: a missing library is an error.
"""
from .binding import (  # noqa: F401
    ZQError,
    gemm_choose_variant,
    gemm_quantizes_in_kernel,
    quant_wait_expired,
    set_in_kernel_quant,
    gemm_stream_plan,
    gemm_stream_k_ranges,
    gemm_w8a16_stream_plan,
    gemm_w8a16_workspace_bytes,
    gemm_variant_name,
    gemm_workspace_bytes,
    gemm_quant_workspace_bytes,
    new_workspace,
    zq_workspace_init,
    WORKSPACE_FIXED_BYTES,
    force_gemm_variant,
    lib,
    tune_clear,
    tune_count,
    tune_set,
    lib_path,
    version,
    zq_dequantize_acc,
    zq_gelu_quant_tokenwise,
    zq_gemm_gelu_quant_tokenwise,
    zq_gemm_i8_dequant,
    zq_gemm_i8_dequant_static,
    STATIC_SCRATCH_BYTES,
    zq_gemm_w4a8_dequant,
    zq_gemm_w8a16_dequant,
    zq_layernorm_quant_tokenwise,
    zq_quantize_tokenwise,
    zq_quantize_weight_groupwise,
    zq_probe_mfma_i8,
    zq_probe_mfma_i8_tile_traffic,
    zq_probe_read_stream,
)
