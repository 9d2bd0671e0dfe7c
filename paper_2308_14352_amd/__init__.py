"""MI355X-native mixed-bitwidth MoE layer forward (EdgeMoE's data-parallel hot path).

`binding` mirrors the C ABI in include/moeq.h; `build` compiles the HIP library in-tree.
"""
from . import binding  # noqa: F401
from .binding import (MOEQ_ACT_RELU, MOEQ_ACT_SWIGLU, MOEQ_BF16, MOEQ_F32, MOEQ_IN_CANONICAL, MOEQ_IN_STREAM,  # noqa: F401
                      MOEQ_OUT_CANONICAL, MOEQ_PATH_STREAM, moe_prepare_in, moe_unprepare_in, moe_stream_bytes,
                      MOEQ_OUT_COLUMNS, MOEQ_PATH_GROUPED_GEMM, MOEQ_PATH_ONE_KERNEL, MOEQ_PATH_ONE_KERNEL_MX,
                      MOEQ_PATH_TWO_KERNELS, Layer, MoeqError, PackedExpert, moe_dequantize, moe_expert_ffn_q,
                      moe_layer_forward, moe_layer_forward_routed, moe_layer_table_bytes, moe_packed_bytes, moe_prepare_out,
                      moe_quantize_pack, moe_router_topk, moe_unpack_codes, moe_unprepare_out)
