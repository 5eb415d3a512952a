"""HiFT step library for AMD MI355X: thin Python binding over the C ABI in include/hift.h.

The shared library libhift.so must have been built (python -m paper_2401_15207_amd.build, or
__graft_entry__.build()); importing this package fails loudly when it is missing.
"""
from .binding import (HiftError, HiftModel, lib, group_count, group_order, tensor_list, query_bytes, memory_report, lr_at_cycle,
                      kernel_gemm, kernel_packed_bytes, kernel_pack_b, kernel_gemm_packed, kernel_optimizer, kernel_norm_fwd, kernel_packed_workspace_bytes, kernel_gemm_packed_ws, kernel_gemm_packed_static, kernel_linear_fused, kernel_gemm_packed_rowsq, kernel_row_sumsq, kernel_linear_norm_fused, kernel_linear_gelu, EPILOGUE_SWIGLU, EPILOGUE_ROPE, EPILOGUE_SWIGLU_BWD, UNFUSED_EPILOGUES, UNFUSED_ATTENTION, UNFUSED_NORM, UNSHARED_LAST_ROUND, kernel_attention_fwd, kernel_attention_bwd, kernel_cross_entropy, LIB_PATH)

__all__ = ["HiftError", "HiftModel", "lib", "group_count", "group_order", "tensor_list", "query_bytes", "memory_report", "lr_at_cycle",
           "kernel_gemm", "kernel_packed_bytes", "kernel_pack_b", "kernel_gemm_packed", "kernel_optimizer", "kernel_norm_fwd", "kernel_packed_workspace_bytes", "kernel_gemm_packed_ws", "kernel_gemm_packed_static", "kernel_linear_fused", "kernel_gemm_packed_rowsq", "kernel_row_sumsq", "kernel_linear_norm_fused", "kernel_linear_gelu", "EPILOGUE_SWIGLU", "EPILOGUE_ROPE", "EPILOGUE_SWIGLU_BWD", "UNFUSED_EPILOGUES", "UNFUSED_ATTENTION", "UNFUSED_NORM", "UNSHARED_LAST_ROUND", "kernel_attention_fwd", "kernel_attention_bwd", "kernel_cross_entropy", "LIB_PATH"]
