"""MI355X (gfx950) block-sparse prefill attention: thin Python binding over the
C-ABI library `libsparse_prefill.so` (hand-written HIP kernels).

The binding only marshals arguments: every step of the path runs in the HIP
kernels.  PyTorch supplies device memory and the current stream.
"""
from .binding import (SpaError, attn, attn_vt, check_lists, fused, library_path, load_library, pool, row_capacity, select,
                      select_static, topk_from_scores, transpose_v, value_norms, workspace_bytes)

__all__ = ["SpaError", "attn", "attn_vt", "check_lists", "fused", "library_path", "load_library", "pool", "row_capacity",
           "select", "select_static", "topk_from_scores", "transpose_v", "value_norms", "workspace_bytes"]
