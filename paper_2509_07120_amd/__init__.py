"""Block-sparse global attention for MI355X (gfx950): Python binding of libbsga.so."""
from .block import GlobalAttentionBlock  # noqa: F401
from .binding import (  # noqa: F401
    BSGA_BF16,
    BSGA_FP32,
    BsgaError,
    EXPORTED_SYMBOLS,
    LIB_PATH,
    bsga_attn_workspace_bytes,
    bsga_dense_attn,
    bsga_gather_tokens,
    bsga_pool,
    bsga_pool_qk,
    bsga_select_blocks,
    bsga_select_workspace_bytes,
    bsga_sparse_attn,
    lib,
    num_blocks,
    SpecialTokenPlan,
    sparse_global_attention,
    sparse_global_attention_special,
)
