"""CPU oracle for the FlashOmni attention path -- TEST INFRASTRUCTURE ONLY.

A plain fp64 restatement of what Algorithm 1 computes (two-pass softmax over the kept
key blocks, raw copy for cached query blocks) plus the symbol packing of Section 3.3.
Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the product package never does, and the two share no code.

`gemm_q` and `gemm_o` are the same kind of restatement for the sparse query and output projections
(Section 3.5), `update_symbols` for the symbol generation of an Update step (Section 3.3, Equation 1),
`op_reuse` for the Taylor-series forecast of cached features.

Parity status: every function here is pinned by the CPU test-suite (printed packing
example, textbook dense attention, closed forms, brute force).  Numerical parity with
the authors' own kernel is unpinned: the paper prints no attention outputs.
"""
from .gemm_q import gemm_q, rms_norm, rope, computed_flops as gemm_q_flops  # noqa: F401
from .gemm_o import gemm_o, gemm_o_reuse, reduced_heads as gemm_o_segments, speedup_model as gemm_o_speedup_model  # noqa: F401
from .op_reuse import taylor_coefficients, taylor_update, op_reuse, attention_with_forecast  # noqa: F401
from .symbols import (  # noqa: F401
    update_symbols, compressed_map, caching_metrics, cached_set, skipped_set, contribution_on_query_axis,
)
from .reference import (  # noqa: F401
    pack_symbols,
    unpack_symbols,
    expand_granularity,
    sparse_attention,
    sparse_attention_blocks,
    count_pairs,
    sparsity,
    num_threads,
)
