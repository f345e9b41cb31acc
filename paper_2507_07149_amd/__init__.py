"""MI355X-native DAF activation quantize/pack: thin Python face of libdaf.so.

The three entry points mirror the C ABI in include/daf.h one to one; Python only marshals
arguments.  PyTorch supplies device memory and streams.  There is no CPU fallback: if the
HIP library has not been built, importing `binding` raises.
"""
from .binding import (BF16, F16, F32, REDUCE_ATOMIC, REDUCE_TWO_PASS, STATIC_SCRATCH_BYTES, DafError, Plan, daf_group_minmax, daf_minmax,
                      daf_minmax_workspace, daf_plan, daf_quantize_pack, daf_quantize_pack_batch, daf_quantize_pack_metrics, daf_quantize_pack_static, daf_relu_quantize_pack, daf_linear_quantize_pack, daf_select_bits, daf_select_bits_from_scale,
                      daf_select_bits_workspace, daf_unpack_dequantize, daf_unpack_dequantize_batch, daf_unpack_matmul_grad_weight, daf_unpack_matmul_workspace_bytes,
                      daf_unpack_relu_backward, dequantize_items, dtype_id, lib_path, load_library, quantize_items,
                      rand_bits)

__all__ = ["F32", "F16", "BF16", "REDUCE_TWO_PASS", "REDUCE_ATOMIC", "STATIC_SCRATCH_BYTES", "DafError", "Plan", "daf_plan",
           "daf_quantize_pack", "daf_quantize_pack_static", "daf_unpack_dequantize", "daf_minmax", "daf_minmax_workspace", "daf_group_minmax",
           "daf_select_bits", "daf_select_bits_from_scale", "daf_select_bits_workspace", "daf_quantize_pack_metrics", "daf_relu_quantize_pack", "daf_linear_quantize_pack", "daf_quantize_pack_batch", "daf_unpack_dequantize_batch", "quantize_items",
           "dequantize_items", "daf_unpack_relu_backward", "daf_unpack_matmul_grad_weight", "daf_unpack_matmul_workspace_bytes", "dtype_id",
           "lib_path", "load_library", "rand_bits"]
