"""Correspondence-structured Q/K/V generator for the five benchmark shapes and a higher-resolution one.

Token layout per frame (paper, Sec. 3.1 and Fig. 2): one camera token, four
register tokens, then the patch tokens of a 14x14-pixel patch grid
(518x518 px -> 37x37 = 1369 patches; 518x392 px -> 37x28 = 1036 patches).
Global attention runs over the concatenation of all frames' tokens.

The values are synthetic stand-ins for real activations: every head draws a
pool of latent unit vectors; each patch token is tied to one latent, so tokens
in different frames that share a latent behave like multi-view
correspondences.  From the third shape on, each latent is visible only in a
random subset of frames (partial view overlap).

Nothing here computes any part of the attention method.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np

HEAD_DIM = 64
N_SPECIAL = 5  # 1 camera + 4 register tokens per frame


@dataclass(frozen=True)
class WorkloadConfig:
    cfg_id: int
    name: str
    frames: int
    patches_per_frame: int
    heads: int
    block: int
    dtype: str  # "fp32" or "bf16"
    n_latents: int
    visibility: float  # probability that a latent is visible in a frame (1.0 = always)
    taus: Tuple[float, ...]

    @property
    def tokens_per_frame(self) -> int:
        return N_SPECIAL + self.patches_per_frame

    @property
    def n_tokens(self) -> int:
        return self.frames * self.tokens_per_frame

    @property
    def n_blocks(self) -> int:
        return num_blocks(self.n_tokens, self.block)


def num_blocks(n_tokens: int, block: int) -> int:
    return (n_tokens + block - 1) // block


CONFIGS: Dict[int, WorkloadConfig] = {
    1: WorkloadConfig(1, "2 frames fp32 b64", 2, 37 * 37, 16, 64, "fp32", 2000, 1.0, (0.9,)),
    2: WorkloadConfig(2, "8 frames bf16 b64", 8, 37 * 37, 16, 64, "bf16", 2000, 1.0, (0.8, 0.9, 0.95, 1.0)),
    3: WorkloadConfig(3, "32 frames bf16 b128", 32, 37 * 37, 16, 128, "bf16", 8000, 0.3, (0.9,)),
    4: WorkloadConfig(4, "100 frames bf16 b128", 100, 37 * 37, 16, 128, "bf16", 8000, 0.3, (0.8, 0.9, 0.95)),
    5: WorkloadConfig(5, "300 frames 518x392 bf16 b128", 300, 37 * 28, 16, 128, "bf16", 20000, 0.2, (0.9,)),
    # Higher-resolution input (the paper's discussion: doubling the image side gives four times the
    # patch tokens per frame and sixteen times the global-attention cost).  1036x1036 px -> 74x74
    # patches per frame; 25 frames give about the token count of the 100-frame shape, at a quarter of
    # the frames and four times the tokens per frame (latent pool scaled with the patches per frame).
    6: WorkloadConfig(6, "25 frames 1036x1036 bf16 b128", 25, 74 * 74, 16, 128, "bf16", 32000, 0.3, (0.9,)),
}


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 array of bfloat16 bit patterns (round to nearest even)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> the float32 values they denote (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _head_rng(cfg: WorkloadConfig, head: int, base_seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(base_seed + 1000 * cfg.cfg_id + head))


def generate_head(cfg: WorkloadConfig, head: int, base_seed: int = 0, frames: int | None = None):
    """Q, K, V of one head as float32 arrays [N, 64] holding values already
    rounded to the config's dtype (bf16 values are exactly representable in
    float32).  `frames` overrides the frame count (same per-frame recipe)."""
    n_frames = cfg.frames if frames is None else frames
    rng = _head_rng(cfg, head, base_seed)
    T = cfg.tokens_per_frame
    P = cfg.patches_per_frame
    N = n_frames * T
    z = rng.standard_normal((cfg.n_latents, HEAD_DIM), dtype=np.float32)
    z /= np.linalg.norm(z, axis=1, keepdims=True)

    latent = np.empty((n_frames, P), dtype=np.int64)
    if cfg.visibility >= 1.0:
        latent[:] = rng.integers(0, cfg.n_latents, size=(n_frames, P))
    else:
        visible = rng.random((n_frames, cfg.n_latents)) < cfg.visibility
        for f in range(n_frames):
            ids = np.flatnonzero(visible[f])
            if ids.size == 0:  # degenerate draw: fall back to the whole pool
                ids = np.arange(cfg.n_latents)
            latent[f] = ids[rng.integers(0, ids.size, size=P)]

    q = rng.standard_normal((N, HEAD_DIM), dtype=np.float32)
    k = rng.standard_normal((N, HEAD_DIM), dtype=np.float32)
    v = rng.standard_normal((N, HEAD_DIM), dtype=np.float32)
    q3 = q.reshape(n_frames, T, HEAD_DIM)
    k3 = k.reshape(n_frames, T, HEAD_DIM)
    zt = z[latent]  # [frames, P, 64]
    # patch tokens: 4*z + N(0, 0.5^2); special tokens stay N(0, 1)
    q3[:, N_SPECIAL:, :] = 4.0 * zt + 0.5 * q3[:, N_SPECIAL:, :]
    k3[:, N_SPECIAL:, :] = 4.0 * zt + 0.5 * k3[:, N_SPECIAL:, :]
    if cfg.dtype == "bf16":
        q = bf16_bits_to_f32(round_to_bf16_bits(q))
        k = bf16_bits_to_f32(round_to_bf16_bits(k))
        v = bf16_bits_to_f32(round_to_bf16_bits(v))
    return q, k, v


def generate(cfg: WorkloadConfig, base_seed: int = 0, heads: int | None = None, frames: int | None = None):
    """All heads stacked: three float32 arrays [H, N, 64] (values rounded to cfg.dtype)."""
    H = cfg.heads if heads is None else heads
    n_frames = cfg.frames if frames is None else frames
    N = n_frames * cfg.tokens_per_frame
    q = np.empty((H, N, HEAD_DIM), dtype=np.float32)
    k = np.empty_like(q)
    v = np.empty_like(q)
    def fill(h):
        q[h], k[h], v[h] = generate_head(cfg, h, base_seed, frames)

    if H > 1 and N >= 20000:  # numpy's generators release the GIL on large fills
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(8, H)) as pool:
            list(pool.map(fill, range(H)))
    else:
        for h in range(H):
            fill(h)
    return q, k, v
