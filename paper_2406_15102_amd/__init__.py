"""MI355X-native HLQ backward pass (arXiv 2406.15102): thin Python binding over the C-ABI HIP library.

``binding`` mirrors ``include/hlq.h`` one to one; ``workloads`` draws the seeded synthetic inputs.
"""
from . import workloads  # noqa: F401
from .binding import (  # noqa: F401
    HLQ_BF16, HLQ_F32, HLQ_BITS_4, HLQ_BITS_4_PACKED, HLQ_BITS_8, HLQ_FLAG_GW_INT8, HLQ_FLAG_GX_8BIT,
    HLQ_FLAG_GX_UNPACKED, HLQ_FLAG_ROUND_MANTISSA, HLQ_FLAG_SEPARATE_PRODUCTS, HLQ_BITS_ROUND_MANTISSA, HLQ_BASIS_ROUND_MANTISSA, HLQ_FLAG_GW_SEQUENCY, HLQ_BASIS_NATURAL, HLQ_BASIS_SEQUENCY, hlq_hla_project_basis,
    hlq_hla_quantize_basis, HlqError, hlq_compress_act_int8, hlq_hla_quantize,
    hlq_hla_quantize_workspace_bytes, hlq_gemm_workspace_bytes, hlq_linear_backward_mode, hlq_linear_backward_cached, hlq_weight_code_bits, hlq_workspace_bytes_mode, exported_symbols, hlq_bf16_gemm_nt, hlq_compress_act, hlq_hla_project,
    hlq_int8_gemm_nt, hlq_int4_gemm_nt, hlq_linear_backward, hlq_mfma_probe, hlq_linear_backward_ex, hlq_quantize_g, hlq_quantize_w,
    hlq_quantize_w_workspace_bytes, hlq_status_str, hlq_version, hlq_workspace_bytes, lib,
    hlq_conv_geom, hlq_conv_sizes, hlq_im2col, hlq_col2im, hlq_conv_workspace_bytes, hlq_conv2d_backward,
    hlq_conv_compress_act, hlq_conv_compress_act_int8, hlq_backward_products, hlq_backward_products_workspace_bytes,
    hlq_set_workspace, hlq_quantize_w_static, hlq_compress_act_int4, HLQ_FLAG_XC_INT4, hlq_backward_products_plan, hlq_set_option, HLQ_OPT_PERSISTENT_PRODUCTS, HLQ_OPT_SHARED_G_READ, HLQ_OPT_DIRECT_TO_LDS, HLQ_OPT_PLAN_TILE, HLQ_OPT_PLAN_SPLITS, HLQ_OPT_TAIL_TILES, HLQ_OPT_FRONT_INTERLEAVE,
)
