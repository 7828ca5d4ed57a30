"""MI355X-native two-stage dynamic sparse attention (DSV hot path) behind a C ABI.

The Python layer only marshals arguments: every step of the path runs in the HIP kernels of
libdsv.so.  There is no CPU or PyTorch fallback; a missing library is an error.
"""
from .binding import (  # noqa: F401
    DsvError,
    Problem,
    library_path,
    load_library,
    version,
    idx_offsets,
    lowrank_topk,
    lowrank_topk_workspace,
    lowrank_topk_noalloc,
    lowrank_topk_noalloc_max_bytes,
    lowrank_topk_t,
    lowrank_topk_t_workspace,
    sparse_attn_fwd,
    sparse_attn_fwd_workspace,
    sparse_attn_bwd,
    sparse_attn_bwd_workspace,
    sparse_attn_bwd_dq,
    sparse_attn_bwd_dq_workspace,
    sparse_attn_bwd_dkdv_workspace,
    sparse_attn_bwd_t,
    sparse_attn_bwd_t_workspace,
    idx_transpose,
    idx_transpose_workspace,
    sparse_attn_bwd_dkdv,
    idx_validate,
    lowrank_project,
    lowrank_scores_rows,
    kernel_timing,
    kernel_ms,
    KERNEL_SPANS,
    EXPORTED_SYMBOLS,
)
