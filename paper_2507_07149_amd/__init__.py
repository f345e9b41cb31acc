"""MI355X-native DAF activation quantize/pack: thin Python face of libdaf.so.

The three entry points mirror the C ABI in include/daf.h one to one; Python only marshals
arguments.  PyTorch supplies device memory and streams.  There is no CPU fallback: if the
HIP library has not been built, importing `binding` raises.
"""
from .binding import (BF16, F16, F32, DafError, Plan, daf_plan, daf_quantize_pack, daf_unpack_dequantize,
                      dtype_id, lib_path, load_library, rand_bits)

__all__ = ["F32", "F16", "BF16", "DafError", "Plan", "daf_plan", "daf_quantize_pack",
           "daf_unpack_dequantize", "dtype_id", "lib_path", "load_library", "rand_bits"]
