"""Randomised GPU parity sweeps: shapes, block sizes, split points, densities and thresholds drawn
from a seeded generator, every case checked against the oracle.  They complement the hand-picked
cases of the other GPU tests: no shape here is special, so an indexing slip that the picked shapes
happen to avoid has a good chance of showing up.

Attention (Sec. 4.1 Eq. (2), blocks as in Sec. 4.2 when the sequence is split): random masks with a
full row, possibly an empty row, possibly key blocks of 64 under query blocks of 128; a few cases are
large enough for the launch-order path.  Selection (Sec. 4.1, selecting blocks): random pooled vectors
with exact ties, every combination of CDF threshold, top-k floor, score scale and forced rows / columns.
"""
import numpy as np
import pytest
import torch

from oracle import bsga_oracle as O
from tests.helpers import bf16_bars_ok, bits_to_mask, lists_to_mask, to_device, unexcused_mask_mismatches
from workload import bf16_bits_to_f32, round_to_bf16_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import paper_2509_07120_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pkg


def _attention_case(seed):
    rng = np.random.default_rng(seed)
    b = int(rng.choice([64, 128]))
    bk = 64 if (b == 128 and rng.random() < 0.4) else b
    big = rng.random() < 0.15                     # enough rows for the launch-order path
    H = 8 if big else int(rng.integers(1, 4))
    N = int(rng.integers(128 * b + 1, 128 * b + 2000)) if big else int(rng.integers(1, 1800))
    n_first = N if rng.random() < 0.4 else int(rng.integers(0, N + 1))
    density = float(rng.choice([0.03, 0.1, 0.3, 0.9, 1.0]))
    q, k, v = (rng.standard_normal((H, N, 64)).astype(np.float32) for _ in range(3))
    q *= float(rng.choice([0.3, 1.0, 2.0]))
    v *= 0.25
    q, k, v = (bf16_bits_to_f32(round_to_bf16_bits(x)) for x in (q, k, v))
    nbq, nbk = len(O.block_ranges(N, b, n_first)), len(O.block_ranges(N, bk, n_first))
    mask = rng.random((H, nbq, nbk)) < density
    if nbq > 2:
        mask[:, rng.integers(0, nbq), :] = True
    empty = int(rng.integers(0, nbq)) if (nbq > 3 and rng.random() < 0.5) else None
    for h in range(H):
        for I in range(nbq):
            if not mask[h, I].any():
                mask[h, I, rng.integers(0, nbk)] = True
    if empty is not None:
        mask[:, empty, :] = False
    sample = None
    if big:
        sample = sorted(set([0, nbq - 1] + [int(x) for x in rng.integers(0, nbq, 6)]) - {empty})
    return b, bk, n_first, q, k, v, mask, empty, sample


@pytest.mark.parametrize("seed", range(40))
def test_random_attention_case(B, seed):
    b, bk, n_first, q, k, v, mask, empty, sample = _attention_case(seed)
    H, N, _ = q.shape
    idx, cnt = O.mask_to_index_lists(mask)
    tidx, tcnt = torch.from_numpy(np.where(idx < 0, 0, idx)).cuda(), torch.from_numpy(cnt).cuda()
    tq, tk, tv = (to_device(x, "bf16") for x in (q, k, v))
    print(f"b={b} bk={bk} H={H} N={N} n_first={n_first} kept={mask.mean():.2f} empty={empty}", flush=True)
    out = B.bsga_sparse_attn_split(tq, tk, tv, b, n_first, tidx, tcnt, block_k=bk)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    ranges = O.block_ranges(N, b, n_first)
    want_mask = mask.copy()
    if empty is not None:                         # a row that keeps nothing is zeros by definition
        lo, hi = ranges[empty]
        assert (out[:, lo:hi].float() == 0).all()
        want_mask[:, empty, 0] = True             # (the oracle has no empty rows; that row is not compared)
    want = O.sparse_attention(q, k, v, want_mask, b, q_blocks=sample, b_k=bk, n_first=n_first)
    if empty is not None:
        want[:, ranges[empty][0]:ranges[empty][1]] = np.nan
    ok, ratio, mean = bf16_bars_ok(out, want)
    assert ok, (ratio, mean)


@pytest.mark.parametrize("seed", range(60))
def test_random_selection_case(B, seed):
    rng = np.random.default_rng(1000 + seed)
    H = int(rng.integers(1, 4))
    nbq = int(rng.integers(1, 400))
    nbk = int(rng.integers(1, 400)) if rng.random() < 0.5 else nbq
    if rng.random() < 0.1:
        nbk = int(rng.integers(1000, 2600))
    qp = rng.standard_normal((H, nbq, 64)) * float(rng.choice([0.05, 0.3, 1.0, 3.0, 10.0]))
    kp = rng.standard_normal((H, nbk, 64))
    if rng.random() < 0.2:
        kp[:, rng.integers(0, nbk)] = kp[:, 0]    # two key blocks with exactly equal scores in every row
    tau = float(rng.choice([0.0, 0.3, 0.5, 0.9, 0.99, 0.999999, 1.0]))
    rho = float(rng.choice([1.0, 0.9, 0.75, 0.5, 0.1, 0.0]))
    scale = float(rng.choice([0.125, 1.0, 0.01]))
    fq = (rng.random(nbq) < 0.1).astype(np.uint8) if rng.random() < 0.3 else None
    fk = (rng.random(nbk) < 0.1).astype(np.uint8) if rng.random() < 0.3 else None
    print(f"H={H} nbq={nbq} nbk={nbk} tau={tau} rho={rho} scale={scale} force_q={fq is not None} force_k={fk is not None}",
          flush=True)
    bits, idx, cnt = B.bsga_select_blocks(torch.from_numpy(qp).cuda(), torch.from_numpy(kp).cuda(), tau, rho,
                                          score_scale=scale,
                                          force_q=None if fq is None else torch.from_numpy(fq).cuda(),
                                          force_k=None if fk is None else torch.from_numpy(fk).cuda())
    torch.cuda.synchronize()
    got = bits_to_mask(bits, nbk)
    assert (got == lists_to_mask(idx, cnt, nbk)).all()          # the two output forms agree
    counts, lists = cnt.cpu().numpy(), idx.cpu().numpy()
    assert (counts == got.sum(-1)).all()
    for h in range(H):
        for I in range(nbq):
            assert (np.diff(lists[h, I, :counts[h, I]]) > 0).all()  # ascending, no duplicates
    logits = O.block_logits(qp, kp, scale)
    probs = O.block_softmax(logits)
    want = O.select_blocks(probs, tau, rho, fq, fk)
    if fq is not None:
        assert got[:, fq.astype(bool), :].all()
    if fk is not None:
        assert got[:, :, fk.astype(bool)].all()
    unexcused, excused = unexcused_mask_mismatches(got, want, logits, probs, tau, rho)
    assert unexcused == 0, (unexcused, excused)
