"""The global-attention transformer block (projections -> bsga library -> output projection -> MLP)
on random weights: the attention part against the oracle on the block's own q, k, v, and the torch
plumbing around it (layouts, token permutation, residuals) against an fp64 numpy chain."""
import numpy as np
import pytest
import torch

from oracle import bsga_oracle as O
from tests.helpers import attn_errors

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import paper_2509_07120_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pkg


def _f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def _layer_norm(x, w, b, eps=1e-5):
    mu = x.mean(-1, keepdims=True)
    var = ((x - mu) ** 2).mean(-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * w + b


def _gelu(x):
    from scipy.special import erf
    return 0.5 * x * (1.0 + erf(x / np.sqrt(2.0)))


@pytest.mark.parametrize("use_special,tau,rho", [(True, 0.9, 1.0), (False, 0.0, 0.5), (True, 1.0, 1.0)])
def test_block_against_fp64_chain(B, use_special, tau, rho):
    frames, per_frame, D, H, b = 4, 1374, 1024, 16, 128
    N = frames * per_frame
    special = (torch.arange(N) % per_frame) < 5
    blk = B.GlobalAttentionBlock(D, H, b, tau, rho, special=special if use_special else None, seed=3)
    g = torch.Generator().manual_seed(7)
    x = torch.randn(N, D, generator=g).to(torch.bfloat16).cuda()
    y = blk(x)
    torch.cuda.synchronize()
    q, k, v, o = (_f64(blk.last[n]) for n in ("q", "k", "v", "o"))

    # 1. attention on the block's own q, k, v (working order) against the oracle
    if use_special:
        n_patch = int((~special).sum())
        npb = -(-n_patch // b)                            # the last patch block is ragged
        patch_idx = np.arange(n_patch)                    # working order: every patch token first,
        special_idx = np.arange(n_patch, N)               # then every special token
        if tau >= 1.0:
            want = O.dense_attention(q, k, v)
        else:
            want, _ = O.special_token_attention(q, k, v, patch_idx, special_idx, b, tau, rho, heads=[0, 5],
                                                patch_blocks=[0, 1, npb // 2, npb - 1])
    else:
        mask = O.predict_mask(q[[0, 5]], k[[0, 5]], b, tau, rho)
        want = np.full_like(o, np.nan)
        want[[0, 5]] = O.sparse_attention(q[[0, 5]], k[[0, 5]], v[[0, 5]], mask, b)
    mx, mean = attn_errors(blk.last["o"], want)
    assert mx <= 1e-2 and mean <= 1e-3, (mx, mean)

    # 2. projections and layout: q, k, v against fp64 (bf16 GEMM outputs of O(1) values)
    xf = _f64(x)
    h = _layer_norm(xf, _f64(blk.ln1.weight), _f64(blk.ln1.bias))
    order = _f64(blk.plan.perm).astype(np.int64) if use_special else np.arange(N)
    qkv = h[order] @ _f64(blk.w_qkv).T + _f64(blk.b_qkv)
    qkv = qkv.reshape(N, 3, H, 64).transpose(1, 2, 0, 3)
    for got, ref in ((q, qkv[0]), (k, qkv[1]), (v, qkv[2])):
        assert np.abs(got - ref).max() <= 0.08 and np.abs(got - ref).mean() <= 0.01

    # 3. output projection, un-permutation, residuals, MLP: fp64 chain continued from the GPU's o
    yo = o.transpose(1, 0, 2).reshape(N, D) @ _f64(blk.w_out).T + _f64(blk.b_out)
    inv = np.empty(N, dtype=np.int64)
    inv[order] = np.arange(N)
    x1 = xf + yo[inv]
    h2 = _layer_norm(x1, _f64(blk.ln2.weight), _f64(blk.ln2.bias))
    x2 = x1 + _gelu(h2 @ _f64(blk.w_fc1).T + _f64(blk.b_fc1)) @ _f64(blk.w_fc2).T + _f64(blk.b_fc2)
    err = np.abs(_f64(y) - x2)
    assert err.max() <= 0.15 and err.mean() <= 0.02, (err.max(), err.mean())
