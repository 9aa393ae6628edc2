"""One global-attention transformer block of a VGGT-like aggregator around the bsga library
(Sec. 3.1 for the alternating-attention design, Sec. 4.1 / 4.2 for what replaces the dense global
attention; the appendix "Theoretical FLOPs Reduction" for the block's parts: attention with its
projections plus an MLP with d_ff = 4 d).

Integration shape only: random weights, timing and parity of the data path.  The projections, the
layer norms and the MLP are plain torch ops (library GEMMs); pooling, selection, block-sparse attention
and the token gathers are the bsga kernels.
"""
from __future__ import annotations

from typing import Optional

import torch
import torch.nn.functional as F

from . import binding as B


class GlobalAttentionBlock(torch.nn.Module):
    """x [N, d_model] (all frames' tokens of one scene) -> x + Attn(LN(x)) -> + MLP(LN(.)).

    heads * 64 == d_model.  `special` (bool [N], optional) marks the camera / register tokens: with it
    the block map is predicted on patch tokens only and everything touching a special token stays
    dense (Sec. 4.2); without it all tokens are treated alike.  tau >= 1 with rho = 1 runs the dense
    kernel.
    """

    def __init__(self, d_model: int = 1024, heads: int = 16, block: int = 128, tau: float = 0.9, rho: float = 1.0,
                 special: Optional[torch.Tensor] = None, mlp: bool = True, dtype=torch.bfloat16, device="cuda",
                 seed: int = 0):
        super().__init__()
        assert d_model == heads * 64, "head dimension must be 64"
        g = torch.Generator(device="cpu").manual_seed(seed)

        def w(*shape, scale):
            return torch.nn.Parameter((torch.randn(*shape, generator=g) * scale).to(dtype).to(device), requires_grad=False)

        self.d_model, self.heads, self.block, self.tau, self.rho = d_model, heads, block, tau, rho
        self.w_qkv = w(3 * d_model, d_model, scale=d_model ** -0.5)
        self.b_qkv = w(3 * d_model, scale=0.02)
        self.w_out = w(d_model, d_model, scale=d_model ** -0.5)
        self.b_out = w(d_model, scale=0.02)
        self.ln1 = torch.nn.LayerNorm(d_model, device=device, dtype=dtype)
        self.mlp = mlp
        if mlp:
            self.ln2 = torch.nn.LayerNorm(d_model, device=device, dtype=dtype)
            self.w_fc1 = w(4 * d_model, d_model, scale=d_model ** -0.5)
            self.b_fc1 = w(4 * d_model, scale=0.02)
            self.w_fc2 = w(d_model, 4 * d_model, scale=(4 * d_model) ** -0.5)
            self.b_fc2 = w(d_model, scale=0.02)
        self.plan = None if special is None else B.SpecialTokenPlan(special, block, device)
        self.last = {}  # q, k, v, o of the last call ([H, N, 64], working order), for tests

    @torch.no_grad()
    def attention(self, x: torch.Tensor) -> torch.Tensor:
        N, D = x.shape
        H = self.heads
        h = self.ln1(x)
        if self.plan is not None:  # working order: patch tokens first, special tokens last
            h = h.index_select(0, self.plan.perm.long())
        qkv = F.linear(h, self.w_qkv, self.b_qkv).view(N, 3, H, 64).permute(1, 2, 0, 3).contiguous()  # [3, H, N, 64]
        q, k, v = qkv[0], qkv[1], qkv[2]
        if self.tau >= 1.0 and self.rho >= 1.0:
            o = B.bsga_dense_attn(q, k, v)
        else:
            # with the split, patch tokens and special tokens are blocked separately (n_first = N_p)
            n_first = N if self.plan is None else self.plan.n_patch
            q_pool, k_pool = B.bsga_pool_qk_split(q, k, self.block, n_first)
            fq = None if self.plan is None else self.plan.force_q
            fk = None if self.plan is None else self.plan.force_k
            _, kv_idx, kv_cnt = B.bsga_select_blocks(q_pool, k_pool, self.tau, self.rho, force_q=fq, force_k=fk,
                                                     want_bits=False)
            o = B.bsga_sparse_attn_split(q, k, v, self.block, n_first, kv_idx, kv_cnt)
        self.last = {"q": q, "k": k, "v": v, "o": o}
        y = F.linear(o.permute(1, 0, 2).reshape(N, D), self.w_out, self.b_out)
        if self.plan is not None:
            y = y.index_select(0, self.plan.inverse.long())
        return y

    @torch.no_grad()
    def forward(self, x: torch.Tensor) -> torch.Tensor:
        x = x + self.attention(x)
        if self.mlp:
            x = x + F.linear(F.gelu(F.linear(self.ln2(x), self.w_fc1, self.b_fc1)), self.w_fc2, self.b_fc2)
        return x
