"""MI355X (gfx950) quantized attention forward pass after SageAttention2 (arXiv 2411.10958).

The compute lives in libsageattn.so (hand-written HIP kernels behind the C ABI declared in
include/sage_attn.h); this package is a thin ctypes binding with the same entry-point names.
PyTorch is used only to own device memory and streams.
"""
from .binding import (make_varlen_args, SAGE_MODE_INT4_FP8, SAGE_MODE_INT8_FP8, SAGE_DT_FP16, SAGE_DT_BF16,
                      SageError, lib_path, load_library, sage_attn_workspace_bytes, sage_attn_kv_splits,
                      sage_attn_fwd_ex, sage_attn_prologue, sage_attn_core, sage_attn_fwd, sage_attn_fwd_static,
                      sage_attn_release, sage_attn_quant, sage_attn_kv_stats, sage_attn_kv_stats_update, sage_attn_debug_qk, sage_attn_debug_mfma_fp8, sage_status_string,
                      make_args)

__all__ = [n for n in dir() if n.startswith(("sage_", "SAGE_", "Sage"))] + ["lib_path", "load_library", "make_args", "make_varlen_args"]
