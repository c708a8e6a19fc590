"""SepAttention (SepLLM, arXiv 2412.12094) for AMD MI355X: hand-written HIP kernels behind a C ABI.

`csrc/` holds the kernels and the C entry points declared in include/sepattn.h; `binding.py` is the
ctypes binding with the same names; `build.py` compiles libsepattn.so in-tree with hipcc for gfx950.
"""
from .binding import (  # noqa: F401
    EXPORTS,
    LIB_PATH,
    SEPATTN_BF16,
    SEPATTN_FP32,
    SepattnError,
    SepattnParams,
    SepkvParams,
    load,
    status_string,
    sepattn_mark_separators,
    sepattn_mark_interval,
    sepattn_compact_indices,
    sepattn_mark_compact,
    sepattn_forward,
    sepattn_forward_headwise,
    sepattn_backward_headwise,
    sepattn_doc_bounds,
    sepattn_forward_packed,
    sepattn_backward_packed,
    sepattn_backward,
    sepattn_backward_workspace_bytes,
    sepattn_decode,
    sepattn_decode_noalloc,
    sepkv_evict_window,
    sepkv_fill_from_prefill,
    sepkv_rope_table,
    sepattn_decode_rope,
    sepkv_append,
    KERNEL_IDS,
    sepattn_kernel_name,
    sepattn_profile_begin,
    sepattn_profile_end,
)
