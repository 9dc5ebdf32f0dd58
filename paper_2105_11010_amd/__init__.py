"""SPARQ trimmed convolution-as-GEMM on AMD MI355X (gfx950).

Thin Python front end of ``libsparq.so`` (see ``include/sparq.h``): the names
below are the C entry points, taking torch device tensors as plain buffers.
"""
from .binding import (  # noqa: F401
    LIB_PATH, SparqConvDesc, SparqError, SparqMode, conv_desc, lib, mode, out_rows, strerror,
    sparq_conv_gemm, sparq_conv_gemm_static_ws, sparq_conv_gemm_u8, sparq_conv_plan, sparq_dequant, sparq_pack_weights, sparq_packed_bytes,
    sparq_requant, sparq_trim, sparq_workspace_bytes, sparq_packed_act_bytes, sparq_pack_act, sparq_unpack_act,
    sparq_conv_packed_workspace_bytes, sparq_conv_gemm_packed, sparq_sparse24_packed_bytes, sparq_sparse24_workspace_bytes,
    sparq_pack_weights_sparse24, sparq_conv_gemm_sparse24, sparq_sparse24_plan, sparq_set_tuning,
)

__all__ = ["LIB_PATH", "SparqConvDesc", "SparqError", "SparqMode", "conv_desc", "lib", "mode", "out_rows",
           "strerror", "sparq_conv_gemm", "sparq_conv_gemm_static_ws", "sparq_conv_gemm_u8", "sparq_conv_plan", "sparq_dequant", "sparq_pack_weights",
           "sparq_packed_bytes", "sparq_requant", "sparq_trim", "sparq_workspace_bytes", "sparq_packed_act_bytes", "sparq_pack_act",
           "sparq_unpack_act", "sparq_conv_packed_workspace_bytes", "sparq_conv_gemm_packed", "sparq_sparse24_packed_bytes",
           "sparq_sparse24_workspace_bytes", "sparq_pack_weights_sparse24", "sparq_conv_gemm_sparse24", "sparq_sparse24_plan", "sparq_set_tuning"]
