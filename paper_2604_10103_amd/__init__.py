"""MI355X-native hybrid attention of Hybrid Forcing: HIP kernels behind a C ABI, plus a thin binding.

The shared library is loaded on first use (``binding.load()``); importing the package does
not need a GPU.
"""
from .binding import (  # noqa: F401
    HF_BF16,
    HF_F32,
    HF_PHI_RELU,
    HF_PHI_ELU1,
    HFError,
    hf_config,
    hf_window,
    make_config,
    load,
    lib_path,
    hf_version,
    hf_state_bytes,
    hf_state_init,
    hf_state_fold_linear,
    hf_absorb_evicted,
    hf_absorb_workspace_bytes,
    hf_window_advance,
    hf_select_k,
    hf_workspace_bytes,
    hf_block_select,
    hf_block_select_cached,
    hf_hybrid_attn_fwd,
    hf_rope_window_indices,
    hf_rope_tables,
    hf_rope_apply,
    hf_stream_open_chunk,
    hf_stream_step,
    hf_bwd_workspace_bytes,
    hf_hybrid_attn_bwd,
    hf_hybrid_attn_bwd_saved,
    hf_hybrid_attn_fwd_save,
)
