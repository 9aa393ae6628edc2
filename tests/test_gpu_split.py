"""GPU parity for the entry points that take a sequence split in two separately blocked parts
(Sec. 4.2: patch tokens and special tokens never share a block): pooling and block-sparse
attention against the oracle's block_ranges(N, b, n_first) blocking, with a ragged block in the
middle of the sequence (as query block and as key block) and another at its end."""
import numpy as np
import pytest
import torch

from oracle import bsga_oracle as O
from tests.helpers import attn_errors, to_device
from workload import bf16_bits_to_f32, round_to_bf16_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import paper_2509_07120_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pkg


def _qkv(H, N, seed, dtype, vscale=0.25):
    rng = np.random.default_rng(seed)
    q, k, v = (rng.standard_normal((H, N, 64)).astype(np.float32) for _ in range(3))
    v *= vscale
    if dtype == "bf16":
        q, k, v = (bf16_bits_to_f32(round_to_bf16_bits(x)) for x in (q, k, v))
    return q, k, v


def _lists(mask):
    idx, cnt = O.mask_to_index_lists(mask)
    return torch.from_numpy(np.where(idx < 0, 0, idx)).cuda(), torch.from_numpy(cnt).cuda()


@pytest.mark.parametrize("dtype,b,N,n_first", [("bf16", 128, 1000, 300), ("bf16", 64, 1000, 333), ("fp32", 64, 500, 129),
                                               ("bf16", 128, 700, 700), ("bf16", 128, 700, 0), ("bf16", 128, 640, 256),
                                               ("fp32", 128, 300, 1)])
def test_pool_split_matches_oracle(B, dtype, b, N, n_first):
    q, k, _ = _qkv(3, N, 1, dtype)
    qp, kp = B.bsga_pool_qk_split(to_device(q, dtype), to_device(k, dtype), b, n_first)
    torch.cuda.synchronize()
    want_q, want_k = O.pool_blocks(q, b, n_first), O.pool_blocks(k, b, n_first)
    assert qp.shape == want_q.shape
    if dtype == "bf16":  # block sums of bf16 values are exact in fp64
        np.testing.assert_array_equal(qp.cpu().numpy(), want_q)
        np.testing.assert_array_equal(kp.cpu().numpy(), want_k)
    else:
        np.testing.assert_allclose(qp.cpu().numpy(), want_q, rtol=0, atol=1e-14)
        np.testing.assert_allclose(kp.cpu().numpy(), want_k, rtol=0, atol=1e-14)


@pytest.mark.parametrize("dtype,b,bk,N,n_first", [
    ("bf16", 128, 128, 1000, 300),    # ragged block 2 (44 tokens) inside, ragged end (60)
    ("bf16", 128, 128, 129 + 500, 129),  # one token in the inner ragged block
    ("bf16", 128, 128, 1374 * 2, 1369 * 2),  # two frames: 2738 patch tokens, 10 special tokens
    ("bf16", 128, 64, 1000, 300),     # key blocks of 64: inner ragged key block of 44, query block of 44
    ("bf16", 64, 64, 700, 333),
    ("fp32", 64, 64, 500, 129),
    ("fp32", 128, 128, 500, 300),
    ("bf16", 128, 128, 640, 256),     # no ragged block at all
])
def test_sparse_attn_split_matches_oracle(B, dtype, b, bk, N, n_first):
    H = 2
    q, k, v = _qkv(H, N, N + n_first, dtype)
    nbq, nbk = len(O.block_ranges(N, b, n_first)), len(O.block_ranges(N, bk, n_first))
    assert nbq == B.split_blocks(N, n_first, b) and nbk == B.split_blocks(N, n_first, bk)
    rng = np.random.default_rng(N)
    mask = rng.random((H, nbq, nbk)) < 0.5
    inner = -(-n_first // bk) - 1                      # the ragged key block inside the sequence
    mask[:, :, inner] |= rng.random((H, nbq)) < 0.7
    mask[:, 0, :] = False; mask[:, 0, inner] = True    # a row that sees only that block
    mask[:, nbq - 1, :] = False; mask[:, nbq - 1, [inner, nbk - 1]] = True   # both ragged blocks, nothing else
    mask[:, :, 0] |= ~mask.any(-1)
    idx, cnt = _lists(mask)
    out, lse = B.bsga_sparse_attn_split(to_device(q, dtype), to_device(k, dtype), to_device(v, dtype), b, n_first, idx, cnt,
                                        return_lse=True, block_k=bk)
    torch.cuda.synchronize()
    want, want_lse = O.sparse_attention(q, k, v, mask, b, b_k=bk, n_first=n_first, return_lse=True)
    assert not np.isnan(want).any()
    mx, mean = attn_errors(out, want)
    lim = (1e-2, 1e-3, 2e-2) if dtype == "bf16" else (1e-5, 1e-6, 1e-5)
    assert mx <= lim[0] and mean <= lim[1], (mx, mean)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= lim[2]


def test_split_at_the_end_equals_the_plain_entry_point(B):
    H, N, b = 2, 900, 128
    q, k, v = _qkv(H, N, 5, "bf16")
    nb = O.num_blocks(N, b)
    mask = np.random.default_rng(2).random((H, nb, nb)) < 0.6
    mask[:, :, 0] = True
    idx, cnt = _lists(mask)
    tq, tk, tv = (to_device(x, "bf16") for x in (q, k, v))
    a = B.bsga_sparse_attn(tq, tk, tv, b, idx, cnt)
    c = B.bsga_sparse_attn_split(tq, tk, tv, b, N, idx, cnt)
    torch.cuda.synchronize()
    assert torch.equal(a, c)
