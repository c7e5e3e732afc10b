"""FlashOmni's unified sparse attention kernel, written for AMD MI355X (gfx950).

The product is the C-ABI library built from ``csrc/`` (declared in ``include/sparse_attn.h``);
this package is the thin Python binding over it plus the seeded synthetic workloads.
"""
from . import synth  # noqa: F401
from .binding import (  # noqa: F401
    SparseAttnError,
    library_path,
    load_library,
    sparse_attn_fwd,
    sparse_attn_fwd_noalloc,
    sparse_attn_fwd_timed,
    sparse_attn_fwd_workspace,
    sparse_attn_release_scratch,
    sparse_gemm_q,
    sparse_gemm_o,
    sparse_gemm_o_reuse,
    SparseAttnPlan,
    sparse_gemm_q_norm_rope,
    sparse_symbols_update,
    sparse_attn_fwd_forecast,
    sparse_op_reuse,
    sparse_taylor_coefficients,
    sparse_taylor_update,
    sparse_attn_profile_begin,
    sparse_attn_profile_end,
    sparse_attn_pack_mask,
    sparse_attn_count_kept,
    sparse_attn_workspace_bytes,
    sparse_attn_version,
    sparse_attn_last_error,
)
