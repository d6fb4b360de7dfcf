"""MI355X-native STS hot path: draft-score selection and sparse verification attention.

Thin Python binding over the C-ABI library ``libsts.so`` (hand-written HIP for gfx950).
The functions here marshal arguments only; every step runs in the library's kernels.
There is no CPU fallback: importing works anywhere, calling requires the built library and
a GPU.
"""
from .binding import (STS_BF16, STS_F32, STS_REDUCE_MAX, STS_REDUCE_SUM, STS_SCORES_LOGITS_LSE,
                      STS_SCORES_PROBS, KERNEL_KINDS, PreparedCall, StsError, attn_plan, exported_symbols,
                      library_path, load_library, set_knob, get_knob, KNOBS, prof_enable, prof_read, prof_reset,
                      sts_dense_attn, sts_head_map, sts_select, sts_sparse_attn, sts_sparse_attn_static,
                      sts_select_rows, sts_union_rows, sts_version, STS_STATIC_SCRATCH_BYTES)

__all__ = ["STS_BF16", "STS_F32", "STS_REDUCE_MAX", "STS_REDUCE_SUM", "STS_SCORES_LOGITS_LSE",
           "STS_SCORES_PROBS", "KERNEL_KINDS", "PreparedCall", "StsError", "attn_plan", "exported_symbols",
           "library_path", "load_library", "set_knob", "get_knob", "KNOBS", "prof_enable", "prof_read", "prof_reset",
           "sts_dense_attn", "sts_head_map", "sts_select", "sts_sparse_attn", "sts_sparse_attn_static",
           "sts_select_rows", "sts_union_rows", "sts_version", "STS_STATIC_SCRATCH_BYTES"]
