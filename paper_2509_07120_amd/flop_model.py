"""Closed-form FLOP and speed-up model of a VGGT-like network with block-sparse global attention
(appendix "Theoretical FLOPs Reduction"), and effective-sparsity accounting for block masks.

Conventions of that appendix: only matrix multiplications of the attention and MLP layers count, a
multiply-add counts once, rho is the fraction of query-key interactions that is SKIPPED (rho = 0 is
dense attention).  Readings where the appendix's formulas do not type-check: the MLP term of a
block is per token (t * FLOP_MLP), and the global term carries the number of global blocks L_G.
With d = 1024, 24 encoder + 24 frame-wise blocks (L_F = 48) and L_G = 24 these formulas give the
appendix's table once the ratios are cut (not rounded) to one decimal.

Host-side arithmetic only; nothing here touches the GPU.
"""
from __future__ import annotations

from dataclasses import dataclass


@dataclass(frozen=True)
class ModelShape:
    d: int = 1024          # model dimension of encoder and aggregator
    frame_blocks: int = 48  # L_F: per-frame transformer blocks (24 encoder + 24 frame-wise aggregator)
    global_blocks: int = 24  # L_G: global-attention blocks


def flop_mlp(d: int) -> int:
    """MLP FLOPs per token: d*d_ff + d_ff*d with d_ff = 4d."""
    return 8 * d * d


def flop_attn(t: int, d: int, rho: float) -> float:
    """Self-attention over t tokens: QKV and output projections (4 t d^2) plus the query-key and
    weight-value products (2 t^2 d), of which a fraction rho is skipped."""
    return 4.0 * t * d * d + (1.0 - rho) * 2.0 * t * t * d


def flop_block(t: int, d: int, rho: float = 0.0) -> float:
    """One transformer block over t tokens: attention plus the per-token MLP."""
    return flop_attn(t, d, rho) + t * flop_mlp(d)


def flop_total(n_frames: int, tokens_per_frame: int, rho: float, shape: ModelShape = ModelShape()) -> float:
    """Forward FLOPs: L_F frame-wise blocks on each frame (always dense) + L_G global blocks over
    all n_frames * tokens_per_frame tokens with sparsity rho."""
    frame = shape.frame_blocks * n_frames * flop_block(tokens_per_frame, shape.d, 0.0)
    glob = shape.global_blocks * flop_block(n_frames * tokens_per_frame, shape.d, rho)
    return frame + glob


def theoretical_speedup(n_frames: int, tokens_per_frame: int, rho: float, shape: ModelShape = ModelShape()) -> float:
    """Upper bound of the end-to-end speed-up at sparsity rho: FLOP(dense) / FLOP(rho)."""
    return flop_total(n_frames, tokens_per_frame, 0.0, shape) / flop_total(n_frames, tokens_per_frame, rho, shape)


def attention_only_speedup(sparsity: float) -> float:
    """Upper bound of the attention kernel's own speed-up when a fraction `sparsity` is skipped."""
    return float("inf") if sparsity >= 1.0 else 1.0 / (1.0 - sparsity)


def effective_sparsity(kept_pairs_tokens: float, n_query_tokens: int, n_key_tokens: int) -> float:
    """Fraction of query-key token pairs that is skipped: 1 - computed / total.  `kept_pairs_tokens`
    counts token pairs (valid tokens of each kept block pair, dense special-token rows and columns
    included), so ragged blocks and always-dense parts are accounted for exactly."""
    return 1.0 - float(kept_pairs_tokens) / (float(n_query_tokens) * float(n_key_tokens))


def kept_token_pairs(kv_cnt_rows, last_block_kept_rows, n_tokens: int, block: int) -> int:
    """Token pairs computed by a block-sparse layer over one head.
    kv_cnt_rows[I]         number of kept key blocks of query block I,
    last_block_kept_rows[I] whether the (possibly ragged) last key block is among them."""
    nb = -(-n_tokens // block)
    tail = n_tokens - (nb - 1) * block
    total = 0
    for i in range(nb):
        rows = tail if i == nb - 1 else block
        keys = int(kv_cnt_rows[i]) * block - ((block - tail) if last_block_kept_rows[i] else 0)
        total += rows * keys
    return total
