"""MI355X-native fused decoder step of temporal fusion (Flover): HIP kernels behind a C ABI.

`binding` is argument marshalling over libflover.so; every step of the path runs in the HIP kernels.
"""
from .binding import (Flover, FloverError, StepOut, ReorderOut, lib_path, load_library, k_find_window,
                      k_decode_attention, k_decode_attention_noalloc, k_compact, k_gemm, k_gated_mlp, k_copy_probe, arena_bytes, EXPORTED_SYMBOLS)

__all__ = ["Flover", "FloverError", "StepOut", "ReorderOut", "lib_path", "load_library", "k_find_window",
           "k_decode_attention", "k_decode_attention_noalloc", "k_compact", "k_gemm", "k_gated_mlp", "k_copy_probe", "arena_bytes", "EXPORTED_SYMBOLS"]
