"""MI355X-native SparseD attention: Python face of the C-ABI library libsparsed.so."""
from .binding import (  # noqa: F401
    BlockIndex,
    SparsedError,
    attn_dense,
    attn_sparse,
    index_fill_window,
    index_validate,
    index_window_entries,
    probe_mfma_bf16,
    probe_valu_f32,
    kept_blocks,
    load_library,
    n_dense_steps,
    select_pattern,
    select_pattern_isolated,
    select_pattern_isolated_tokens,
    select_pattern_static,
    STATIC_SCRATCH_BYTES,
    select_workspace_bytes,
    select_workspace_min_bytes,
    version,
)
from .schedule import SparseDLayer  # noqa: F401
