"""GPU parity for rows whose kept keys include a ragged tile (a short last block, or an absent
half-tile with key blocks of 64) while every logit is strongly negative.

The bf16 kernel's first pass takes softmax weights relative to reference 0, so with logits around
-10 .. -20 nats a row's weight sum is tiny (e^-10 .. e^-20 per key).  Tile rows that are not keys
of the listed block must then contribute exactly nothing: a contribution that is removed again
afterwards would leave an error of the size of the true sum.  The cases: N = 129 (one key in the
last block, 127 tile rows that are not keys), the 100-frame workload's tail (56 keys + 72 rows
that are not), rows that keep only the ragged block / the ragged block and one more / a random
half of all blocks, key blocks of 64 with odd counts, and the dense entry point.  Values have the
spread of the workload's (v ~ N(0, 1/16)), so the flat bars of the acceptance rule apply:
max-abs 1e-2, mean-abs 1e-3."""
import numpy as np
import pytest
import torch

from oracle import bsga_oracle as O
from workload import bf16_bits_to_f32, round_to_bf16_bits
from tests.helpers import attn_errors, to_device

pytestmark = pytest.mark.gpu

BF16_MAX, BF16_MEAN = 1e-2, 1e-3


@pytest.fixture(scope="module")
def B():
    import paper_2509_07120_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pkg


def _bf16(x):
    return bf16_bits_to_f32(round_to_bf16_bits(x.astype(np.float32)))


def _shifted_qkv(H, N, shift_nats, seed):
    """q = r + a u, k = r' - a u with |u| = 1: every logit q.k/8 is about -a^2/8 = shift_nats (plus a
    spread of a few nats from the cross terms), far inside the range the first pass accepts."""
    rng = np.random.default_rng(seed)
    a = np.sqrt(8.0 * abs(shift_nats))
    u = np.full(64, 1.0 / 8.0)
    q = _bf16(rng.standard_normal((H, N, 64)) + a * u)
    k = _bf16(rng.standard_normal((H, N, 64)) - a * u)
    v = _bf16(0.25 * rng.standard_normal((H, N, 64)))
    return q, k, v


def _lists(mask):
    idx, cnt = O.mask_to_index_lists(mask)
    return torch.from_numpy(np.where(idx < 0, 0, idx)).cuda(), torch.from_numpy(cnt).cuda()


def _mask_with_ragged_rows(H, nbq, nbk, seed):
    rng = np.random.default_rng(seed)
    mask = rng.random((H, nbq, nbk)) < 0.5
    mask[:, :, nbk - 1] |= rng.random((H, nbq)) < 0.7       # most rows also keep the ragged block
    mask[:, 0, :] = False; mask[:, 0, nbk - 1] = True        # only the ragged block
    if nbq > 1:
        mask[:, 1, :] = False; mask[:, 1, nbk - 1] = True; mask[:, 1, 0] = True   # the ragged block and one more
    mask[:, :, 0] |= ~mask.any(-1)                           # no empty rows
    return mask


@pytest.mark.parametrize("shift", [-10.0, -14.0, -20.0])
@pytest.mark.parametrize("N", [129, 5 * 128 + 56, 128 + 1, 3 * 128 + 108])
def test_sparse_rows_with_ragged_tile_and_negative_logits(B, N, shift):
    H, b = 2, 128
    q, k, v = _shifted_qkv(H, N, shift, seed=int(N - shift))
    nb = O.num_blocks(N, b)
    mask = _mask_with_ragged_rows(H, nb, nb, seed=N)
    idx, cnt = _lists(mask)
    tq, tk, tv = (to_device(x, "bf16") for x in (q, k, v))
    out, lse = B.bsga_sparse_attn(tq, tk, tv, b, idx, cnt, return_lse=True)
    torch.cuda.synchronize()
    want, want_lse = O.sparse_attention(q, k, v, mask, b, return_lse=True)
    assert abs(np.median(want_lse) - shift) < 8.0            # the logits really sit where intended
    mx, mean = attn_errors(out, want)
    assert mx <= BF16_MAX and mean <= BF16_MEAN, (mx, mean)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= 5e-2


@pytest.mark.parametrize("shift", [-10.0, -14.0, -20.0])
@pytest.mark.parametrize("N", [129, 8 * 128 + 56])
def test_dense_with_ragged_tile_and_negative_logits(B, N, shift):
    H = 2
    q, k, v = _shifted_qkv(H, N, shift, seed=int(3 * N - shift))
    tq, tk, tv = (to_device(x, "bf16") for x in (q, k, v))
    out, lse = B.bsga_dense_attn(tq, tk, tv, return_lse=True)
    torch.cuda.synchronize()
    want, want_lse = O.dense_attention(q, k, v, return_lse=True)
    mx, mean = attn_errors(out, want)
    assert mx <= BF16_MAX and mean <= BF16_MEAN, (mx, mean)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= 5e-2


@pytest.mark.parametrize("shift", [-10.0, -14.0, -20.0])
@pytest.mark.parametrize("N", [7 * 64 + 24, 6 * 64 + 1])
def test_key_blocks_of_64_odd_counts_and_negative_logits(B, N, shift):
    """Query blocks of 128, key blocks of 64: a row with an odd number of kept blocks leaves the
    second half of its last tile empty; the last key block is ragged as well."""
    H, bq, bk = 2, 128, 64
    q, k, v = _shifted_qkv(H, N, shift, seed=int(5 * N - shift))
    nbq, nbk = O.num_blocks(N, bq), O.num_blocks(N, bk)
    mask = _mask_with_ragged_rows(H, nbq, nbk, seed=N)
    mask[:, nbq - 1, :] = False; mask[:, nbq - 1, [1, 2, nbk - 1]] = True   # three blocks: an odd count
    idx, cnt = _lists(mask)
    tq, tk, tv = (to_device(x, "bf16") for x in (q, k, v))
    out, lse = B.bsga_sparse_attn(tq, tk, tv, bq, idx, cnt, return_lse=True, block_k=bk)
    torch.cuda.synchronize()
    want, want_lse = O.sparse_attention(q, k, v, mask, bq, b_k=bk, return_lse=True)
    mx, mean = attn_errors(out, want)
    assert mx <= BF16_MAX and mean <= BF16_MEAN, (mx, mean)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= 5e-2


@pytest.mark.parametrize("shift", [-14.0])
def test_block_64_kernel_with_ragged_tile_and_negative_logits(B, shift):
    H, b, N = 2, 64, 5 * 64 + 9
    q, k, v = _shifted_qkv(H, N, shift, seed=99)
    nb = O.num_blocks(N, b)
    mask = _mask_with_ragged_rows(H, nb, nb, seed=N)
    idx, cnt = _lists(mask)
    tq, tk, tv = (to_device(x, "bf16") for x in (q, k, v))
    out = B.bsga_sparse_attn(tq, tk, tv, b, idx, cnt)
    torch.cuda.synchronize()
    mx, mean = attn_errors(out, O.sparse_attention(q, k, v, mask, b))
    assert mx <= BF16_MAX and mean <= BF16_MEAN, (mx, mean)


@pytest.mark.parametrize("logit_nats", [20.0, 30.0])
def test_large_positive_logits_keep_the_flat_bars(B, logit_nats):
    """Logits of +20 .. +30 nats (the size real activations reach) stay inside the first pass's range;
    the softmax scale rides on Q as one more bf16 rounding, which at this size still fits the flat
    bars because most of a logit this large is common to all keys of the row."""
    H, N, b = 2, 5 * 128 + 56, 128
    rng = np.random.default_rng(int(logit_nats))
    a = np.sqrt(8.0 * logit_nats)
    u = np.full(64, 1.0 / 8.0)
    q = _bf16(rng.standard_normal((H, N, 64)) + a * u)
    k = _bf16(rng.standard_normal((H, N, 64)) + a * u)
    v = _bf16(0.25 * rng.standard_normal((H, N, 64)))
    nb = O.num_blocks(N, b)
    mask = _mask_with_ragged_rows(H, nb, nb, seed=7)
    idx, cnt = _lists(mask)
    tq, tk, tv = (to_device(x, "bf16") for x in (q, k, v))
    out, lse = B.bsga_sparse_attn(tq, tk, tv, b, idx, cnt, return_lse=True)
    torch.cuda.synchronize()
    want, want_lse = O.sparse_attention(q, k, v, mask, b, return_lse=True)
    assert np.median(want_lse) > logit_nats
    mx, mean = attn_errors(out, want)
    print(f"logits ~{logit_nats} nats: max={mx:.2e} mean={mean:.2e} lse err={np.abs(lse.cpu().numpy() - want_lse).max():.2e}")
    assert mx <= BF16_MAX and mean <= BF16_MEAN, (mx, mean)
