"""GPU parity for separate query / key block sizes (query blocks of 128 tokens, key blocks of 64):
attention over index lists of half-tile key blocks, and the whole pipeline with Q pooled by 128 and K
by 64, against the oracle."""
import numpy as np
import pytest
import torch

from oracle import bsga_oracle as O
from workload import CONFIGS, generate, bf16_bits_to_f32, round_to_bf16_bits
from tests.helpers import attn_errors, bf16_bars_ok, bits_to_mask, lists_to_mask, to_device, unexcused_mask_mismatches

pytestmark = pytest.mark.gpu
BQ, BK = 128, 64


@pytest.fixture(scope="module")
def B():
    import paper_2509_07120_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pkg


def _rand_bf16(shape, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    return bf16_bits_to_f32(round_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32)))


def _lists(mask):
    idx, cnt = O.mask_to_index_lists(mask)
    idx = np.where(idx < 0, 0, idx)
    return torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda()


@pytest.mark.parametrize("N", [1, 63, 64, 65, 129, 333, 700, 1000])
def test_attention_small_shapes(B, N):
    H = 3
    q, k, v = (_rand_bf16((H, N, 64), 300 + N + i) for i in range(3))
    nbq, nbk = O.num_blocks(N, BQ), O.num_blocks(N, BK)
    rng = np.random.default_rng(N)
    mask = rng.random((H, nbq, nbk)) < 0.5
    mask[:, np.arange(nbq), rng.integers(0, nbk, nbq)] = True      # no empty rows
    mask[0, 0, :] = False; mask[0, 0, nbk - 1] = True              # a row that sees only the ragged last key block
    if nbk > 2:
        mask[1, 0, :] = False; mask[1, 0, [0, nbk - 2, nbk - 1]] = True   # an odd count ending in the ragged block
    idx, cnt = _lists(mask)
    out, lse = B.bsga_sparse_attn(to_device(q, "bf16"), to_device(k, "bf16"), to_device(v, "bf16"), BQ, idx, cnt,
                                  return_lse=True, block_k=BK)
    torch.cuda.synchronize()
    want, want_lse = O.sparse_attention(q, k, v, mask, BQ, return_lse=True, b_k=BK)
    assert bf16_bars_ok(out, want)[0], bf16_bars_ok(out, want)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= 2e-2


def test_every_key_block_listed_equals_dense(B):
    H, N = 2, 900
    q, k, v = (_rand_bf16((H, N, 64), 40 + i) for i in range(3))
    nbq, nbk = O.num_blocks(N, BQ), O.num_blocks(N, BK)
    idx, cnt = _lists(np.ones((H, nbq, nbk), dtype=bool))
    tq, tk, tv = (to_device(x, "bf16") for x in (q, k, v))
    out = B.bsga_sparse_attn(tq, tk, tv, BQ, idx, cnt, block_k=BK)
    dense = B.bsga_dense_attn(tq, tk, tv)
    torch.cuda.synchronize()
    # same tiles in the same order (15 key blocks = 7 full tiles + a half): identical arithmetic
    assert torch.equal(out, dense)


@pytest.mark.parametrize("sign", [+1.0, -1.0])
def test_out_of_range_logits_fall_back(B, sign):
    """Forces the running-max pass with half-tile key blocks (odd counts leave an empty half)."""
    H, N = 2, 600
    u = np.full(64, 1.0 / 8.0, dtype=np.float32)
    rng = np.random.default_rng(5)
    q = bf16_bits_to_f32(round_to_bf16_bits(rng.standard_normal((H, N, 64)).astype(np.float32) + 27.0 * u))
    k = bf16_bits_to_f32(round_to_bf16_bits(rng.standard_normal((H, N, 64)).astype(np.float32) + sign * 27.0 * u))
    v = _rand_bf16((H, N, 64), 6)
    nbq, nbk = O.num_blocks(N, BQ), O.num_blocks(N, BK)
    mask = rng.random((H, nbq, nbk)) < 0.6
    mask[:, :, 0] = True
    mask[0, 1, :] = False; mask[0, 1, [1, 4, nbk - 1]] = True
    idx, cnt = _lists(mask)
    out, lse = B.bsga_sparse_attn(to_device(q, "bf16"), to_device(k, "bf16"), to_device(v, "bf16"), BQ, idx, cnt,
                                  return_lse=True, block_k=BK)
    torch.cuda.synchronize()
    want, want_lse = O.sparse_attention(q, k, v, mask, BQ, return_lse=True, b_k=BK)
    assert abs(np.median(want_lse)) > 80.0
    assert torch.isfinite(out.float()).all()
    mx, mean = attn_errors(out, want)
    assert mx <= 5e-2 and mean <= 5e-3, (mx, mean)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= 0.25


def test_unsupported_pairs_are_refused(B):
    q = torch.zeros((1, 256, 64), dtype=torch.bfloat16, device="cuda")
    idx = torch.zeros((1, 4, 8), dtype=torch.int32, device="cuda")
    cnt = torch.ones((1, 4), dtype=torch.int32, device="cuda")
    with pytest.raises(B.BsgaError):
        B.bsga_sparse_attn(q, q, q, 64, idx, cnt, block_k=128)
    f = q.float()
    with pytest.raises(B.BsgaError):
        B.bsga_sparse_attn(f, f, f, 128, idx, cnt, block_k=64)


@pytest.mark.parametrize("tau,rho", [(0.9, 1.0), (0.0, 0.75)])
def test_pipeline_32_frames(B, tau, rho):
    """Q pooled by 128, K pooled by 64, selection over 344 x 687 blocks, attention; 2 heads of the
    32-frame shape; masks in full, outputs on sampled query blocks."""
    cfg = CONFIGS[3]
    q, k, v = generate(cfg, heads=2)
    N = q.shape[1]
    tq, tk, tv = (to_device(x, cfg.dtype) for x in (q, k, v))
    qp, kp = B.bsga_pool(tq, BQ), B.bsga_pool(tk, BK)
    bits, idx, cnt = B.bsga_select_blocks(qp, kp, tau, rho)
    out = B.bsga_sparse_attn(tq, tk, tv, BQ, idx, cnt, block_k=BK)
    torch.cuda.synchronize()
    nbq, nbk = O.num_blocks(N, BQ), O.num_blocks(N, BK)
    got = bits_to_mask(bits, nbk)
    assert got.shape == (2, nbq, nbk) and (lists_to_mask(idx, cnt, nbk) == got).all()
    logits = O.block_logits(O.pool_blocks(q, BQ), O.pool_blocks(k, BK), 0.125)
    probs = O.block_softmax(logits)
    want_mask = O.select_blocks(probs, tau, rho)
    unexcused, excused = unexcused_mask_mismatches(got, want_mask, logits, probs, tau, rho)
    assert unexcused == 0, (unexcused, excused)
    counts = got.sum(-1)
    blocks = sorted({0, nbq - 1, nbq // 2, int(counts[0].argmin()), int(counts[0].argmax())})
    want = O.sparse_attention(q, k, v, got, BQ, q_blocks=blocks, b_k=BK)
    mx, mean = attn_errors(out, want)
    print(f"asym 128/64 tau={tau} rho={rho}: kept={got.mean():.4f} excused={excused} max={mx:.2e} mean={mean:.2e}")
    assert mx <= 1e-2 and mean <= 1e-3
