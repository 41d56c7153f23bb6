"""MI355X-native any4 / any3 / any2 weight-only GEMM: libany4 (HIP, gfx950) plus a thin binding."""
from .binding import (Any4Error, any4_dequant, any4_gemm, any4_gemm_noalloc, any4_gemm_repacked, any4_gemm_workspace_bytes, any4_pack,
                      any4_repack, any4_repack_bytes,
                      any4_quantize, any4_quantize_max_k, any4_strerror, any4_version, load_library)

__all__ = ["Any4Error", "any4_pack", "any4_dequant", "any4_gemm", "any4_gemm_noalloc", "any4_gemm_workspace_bytes", "any4_repack", "any4_repack_bytes", "any4_gemm_repacked", "any4_quantize", "any4_quantize_max_k",
           "any4_strerror", "any4_version", "load_library"]
