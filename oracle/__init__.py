"""fp64 CPU oracle for the hybrid attention of Hybrid Forcing (test infrastructure).

This package is a checker, not a product path: only tests, the smoke check and the
benchmark's cpu_baseline leg may import it. It shares no code with the HIP library.
"""
from .hybrid_attention import (  # noqa: F401
    PHI_RELU,
    PHI_ELU1,
    phi,
    rope_rotate,
    state_zero,
    state_absorb,
    pool_blocks,
    block_scores,
    select_k,
    select_blocks,
    sparse_attention,
    dense_attention,
    history_readout,
    state_fold_linear,
    hybrid_attention,
)
from .rope import (  # noqa: F401
    default_axis_pairs,
    chunk_temporal_indices,
    window_temporal_indices,
    axis_frequencies,
    rope_tables_3d,
)
from .backward import (  # noqa: F401
    phi_prime,
    sparse_attention_bwd,
    history_readout_bwd,
    hybrid_attention_bwd,
)
