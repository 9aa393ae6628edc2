"""Block-sparse global attention for MI355X (gfx950): Python binding of libbsga.so."""
from .binding import (  # noqa: F401
    BSGA_BF16,
    BSGA_FP32,
    BsgaError,
    EXPORTED_SYMBOLS,
    LIB_PATH,
    bsga_attn_workspace_bytes,
    bsga_dense_attn,
    bsga_pool_qk,
    bsga_select_blocks,
    bsga_select_workspace_bytes,
    bsga_sparse_attn,
    lib,
    num_blocks,
    sparse_global_attention,
)
