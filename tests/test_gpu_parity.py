"""GPU parity: every C-ABI entry point against the fp64 CPU oracle on the same seeded inputs.

Bars: masks and index lists bit-exact (a disagreement is tolerated only on blocks whose logit is
within 1e-5 of the selection cut, and is counted); bf16 attention max-abs <= 1e-2 and
mean-abs <= 1e-3; fp32 attention max-abs <= 1e-5 and mean-abs <= 1e-6 (fp32 accumulation over a
few thousand keys of O(1) values: relative error ~ sqrt(n) * 2^-24 ~ 3e-6 on outputs of
magnitude ~0.1, plus ~1e-6 relative error per weight from fp32 logits)."""
import math

import numpy as np
import pytest
import torch

from oracle import bsga_oracle as O
from workload import CONFIGS, generate
from tests.helpers import (attn_errors, bf16_bars_ok, bits_to_mask, lists_to_mask, oracle_mask_pipeline, to_device,
                           unexcused_mask_mismatches)

pytestmark = pytest.mark.gpu

BF16_MAX, BF16_MEAN = 1e-2, 1e-3
FP32_MAX, FP32_MEAN = 1e-5, 1e-6


@pytest.fixture(scope="module")
def B():
    import paper_2509_07120_amd as pkg
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pkg


def _rand_qkv(H, N, seed, dtype):
    rng = np.random.default_rng(seed)
    q, k, v = (rng.standard_normal((H, N, 64)).astype(np.float32) for _ in range(3))
    if dtype == "bf16":
        from workload import bf16_bits_to_f32, round_to_bf16_bits
        q, k, v = (bf16_bits_to_f32(round_to_bf16_bits(x)) for x in (q, k, v))
    return q, k, v


# ------------------------------------------------------------------------------------- pooling
@pytest.mark.parametrize("dtype,b,N", [("bf16", 64, 10992), ("bf16", 128, 1374 * 3), ("fp32", 64, 2748),
                                       ("fp32", 128, 300), ("bf16", 64, 1), ("bf16", 128, 129)])
def test_pool_matches_oracle(B, dtype, b, N):
    q, k, _ = _rand_qkv(3, N, 1, dtype)
    qp, kp = B.bsga_pool_qk(to_device(q, dtype), to_device(k, dtype), b)
    torch.cuda.synchronize()
    want_q, want_k = O.pool_blocks(q, b), O.pool_blocks(k, b)
    if dtype == "bf16":  # block sums of bf16 values are exact in fp64 -> identical means
        np.testing.assert_array_equal(qp.cpu().numpy(), want_q)
        np.testing.assert_array_equal(kp.cpu().numpy(), want_k)
    else:
        np.testing.assert_allclose(qp.cpu().numpy(), want_q, rtol=0, atol=1e-14)
        np.testing.assert_allclose(kp.cpu().numpy(), want_k, rtol=0, atol=1e-14)


# ------------------------------------------------------------------------------------- selection
def _check_selection(B, q, k, b, tau, rho, dtype, score_scale=None):
    qp, kp, logits, probs, want = oracle_mask_pipeline(q, k, b, tau, rho, score_scale)
    gq, gk = B.bsga_pool_qk(to_device(q, dtype), to_device(k, dtype), b)
    bits, idx, cnt = B.bsga_select_blocks(gq, gk, tau, rho, score_scale)
    torch.cuda.synchronize()
    nbk = want.shape[-1]
    got = bits_to_mask(bits, nbk)
    assert (lists_to_mask(idx, cnt, nbk) == got).all(), "index lists and bit mask disagree"
    assert (cnt.cpu().numpy() == got.sum(-1)).all()
    unexcused, excused = unexcused_mask_mismatches(got, want, logits, probs, tau, rho)
    assert unexcused == 0, f"{unexcused} unexcused mask mismatches ({excused} excused)"
    return got, want, excused


@pytest.mark.parametrize("tau,rho", [(0.8, 1.0), (0.9, 1.0), (0.95, 1.0), (1.0, 1.0), (0.0, 0.75), (0.5, 0.9),
                                     (0.0, 1.0)])
def test_select_config2_shape(B, tau, rho):
    cfg = CONFIGS[2]
    q, k, _ = generate(cfg, heads=4)
    got, want, excused = _check_selection(B, q, k, cfg.block, tau, rho, cfg.dtype)
    if tau >= 1.0:
        assert got.all()
    if tau == 0.0 and rho == 1.0:
        assert (got.sum(-1) == 1).all()
    print(f"tau={tau} rho={rho} kept={got.mean():.4f} excused={excused}")


def test_select_config1_fp32_and_literal_scale(B):
    cfg = CONFIGS[1]
    q, k, _ = generate(cfg, heads=3)
    _check_selection(B, q, k, cfg.block, 0.9, 1.0, cfg.dtype)
    _check_selection(B, q, k, cfg.block, 0.9, 1.0, cfg.dtype, score_scale=1.0)


@pytest.mark.parametrize("nb", [1, 2, 31, 33, 255, 257, 600])
def test_select_sizes_and_structured_rows(B, nb):
    """Random pooled vectors with sharp rows, plus exact ties (duplicate key blocks)."""
    rng = np.random.default_rng(nb)
    H = 2
    qp = rng.standard_normal((H, nb, 64)) * 1.5
    kp = rng.standard_normal((H, nb, 64)) * 1.5
    if nb > 4:
        kp[:, 3] = kp[:, 1]  # exact tie -> lower index ranks first
    for tau, rho in [(0.7, 1.0), (0.3, 0.5), (1.0, 1.0)]:
        logits = O.block_logits(qp, kp, 0.125)
        probs = O.block_softmax(logits)
        want = O.select_blocks(probs, tau, rho)
        bits, idx, cnt = B.bsga_select_blocks(torch.from_numpy(qp).cuda(), torch.from_numpy(kp).cuda(), tau, rho)
        torch.cuda.synchronize()
        got = bits_to_mask(bits, nb)
        assert (lists_to_mask(idx, cnt, nb) == got).all()
        unexcused, excused = unexcused_mask_mismatches(got, want, logits, probs, tau, rho)
        assert unexcused == 0 and excused == 0, (unexcused, excused)


def test_select_tau_one_keeps_blocks_of_negligible_mass(B):
    """tau >= 1 keeps every block by definition (Sec. 4.1, "Selecting Blocks"; tau = 1 must equal
    dense attention): also blocks whose probability is below the rounding of the row's total, here a
    logit spread of 80 .. 200 nats (p down to e^-200)."""
    rng = np.random.default_rng(5)
    nb = 70
    qp = rng.standard_normal((2, nb, 64)) * 6.0
    kp = rng.standard_normal((2, nb, 64)) * 6.0
    logits = O.block_logits(qp, kp, 0.125)
    assert (logits.max(-1) - logits.min(-1)).min() > 60.0
    want = O.select_blocks(O.block_softmax(logits), 1.0, 1.0)
    assert want.all()
    bits, idx, cnt = B.bsga_select_blocks(torch.from_numpy(qp).cuda(), torch.from_numpy(kp).cuda(), 1.0, 1.0)
    torch.cuda.synchronize()
    assert bits_to_mask(bits, nb).all() and (cnt.cpu().numpy() == nb).all()
    # just below 1 the rule is the ranked prefix again, bit-exact with the oracle
    tau = 1.0 - 2.0 ** -40
    probs = O.block_softmax(logits)
    want = O.select_blocks(probs, tau, 1.0)
    bits, idx, cnt = B.bsga_select_blocks(torch.from_numpy(qp).cuda(), torch.from_numpy(kp).cuda(), tau, 1.0)
    torch.cuda.synchronize()
    unexcused, excused = unexcused_mask_mismatches(bits_to_mask(bits, nb), want, logits, probs, tau, 1.0)
    assert unexcused == 0 and not want.all()


@pytest.mark.parametrize("nbk", [4096, 6000, 8192])
def test_select_max_row_length_and_force(B, nbk):
    rng = np.random.default_rng(7)
    nbq = 5
    qp = rng.standard_normal((1, nbq, 64))
    kp = rng.standard_normal((1, nbk, 64))
    fq = np.zeros(nbq, np.uint8); fq[3] = 1
    fk = np.zeros(nbk, np.uint8); fk[[0, 1, 77, nbk - 1]] = 1
    logits = O.block_logits(qp, kp, 0.125)
    probs = O.block_softmax(logits)
    want = O.select_blocks(probs, 0.6, 1.0, fq, fk)
    bits, idx, cnt = B.bsga_select_blocks(torch.from_numpy(qp).cuda(), torch.from_numpy(kp).cuda(), 0.6, 1.0,
                                          force_q=torch.from_numpy(fq).cuda(), force_k=torch.from_numpy(fk).cuda())
    torch.cuda.synchronize()
    got = bits_to_mask(bits, nbk)
    assert (got == want).all()
    assert (lists_to_mask(idx, cnt, nbk) == got).all()
    assert got[0, 3].all()


# ------------------------------------------------------------------------------------- attention
def _random_mask(H, nb, density, seed):
    rng = np.random.default_rng(seed)
    mask = rng.random((H, nb, nb)) < density
    mask[:, np.arange(nb), rng.integers(0, nb, nb)] = True  # no empty rows
    return mask


def _lists(mask):
    idx, cnt = O.mask_to_index_lists(mask)
    idx = np.where(idx < 0, 0, idx)
    return torch.from_numpy(idx).cuda(), torch.from_numpy(cnt).cuda()


@pytest.mark.parametrize("dtype,b,N", [("bf16", 128, 1), ("bf16", 128, 127), ("bf16", 128, 128), ("bf16", 128, 129),
                                       ("bf16", 128, 700), ("bf16", 64, 63), ("bf16", 64, 64), ("bf16", 64, 333),
                                       ("fp32", 64, 200), ("fp32", 128, 300)])
def test_sparse_attention_small_shapes(B, dtype, b, N):
    H = 3
    q, k, v = _rand_qkv(H, N, 100 + N, dtype)
    nb = O.num_blocks(N, b)
    mask = _random_mask(H, nb, 0.5, N)
    if nb > 1:
        mask[0, 0, :] = False; mask[0, 0, nb - 1] = True  # a row that sees only the ragged last block
    idx, cnt = _lists(mask)
    out, lse = B.bsga_sparse_attn(to_device(q, dtype), to_device(k, dtype), to_device(v, dtype), b, idx, cnt,
                                  return_lse=True)
    torch.cuda.synchronize()
    want, want_lse = O.sparse_attention(q, k, v, mask, b, return_lse=True)
    if dtype == "bf16":
        assert bf16_bars_ok(out, want)[0], bf16_bars_ok(out, want)
    else:
        mx, mean = attn_errors(out, want)
        assert mx <= FP32_MAX and mean <= FP32_MEAN, (mx, mean)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= (2e-2 if dtype == "bf16" else 1e-5)


@pytest.mark.parametrize("dtype,N", [("bf16", 700), ("bf16", 128), ("bf16", 5), ("fp32", 200)])
def test_dense_attention_small_shapes(B, dtype, N):
    H = 2
    q, k, v = _rand_qkv(H, N, 200 + N, dtype)
    out, lse = B.bsga_dense_attn(to_device(q, dtype), to_device(k, dtype), to_device(v, dtype), return_lse=True)
    torch.cuda.synchronize()
    want, want_lse = O.dense_attention(q, k, v, return_lse=True)
    if dtype == "bf16":
        assert bf16_bars_ok(out, want)[0], bf16_bars_ok(out, want)
    else:
        mx, mean = attn_errors(out, want)
        assert mx <= FP32_MAX and mean <= FP32_MEAN, (mx, mean)
    assert np.abs(lse.cpu().numpy() - want_lse).max() <= (2e-2 if dtype == "bf16" else 1e-5)


@pytest.mark.parametrize("sign", [+1.0, -1.0])
def test_out_of_range_logits_fall_back_to_online_softmax(B, sign):
    """The bf16 kernel first runs with softmax reference 0 and repeats a workgroup with the
    running-max form when a row sum leaves [2^-80, 2^100].  A common component of 27 along one unit
    direction puts every logit near +-91 nats (+-131 in log2 units), which overflows (+) or flushes
    to zero (-) in the first pass.  Logits this large also amplify the bf16 rounding of the
    pre-scaled Q (relative 2^-9 of a 131-magnitude exponent is ~0.02), hence the wider bars."""
    H, N, b = 2, 600, 128
    rng = np.random.default_rng(11)
    u = np.full(64, 1.0 / 8.0, dtype=np.float32)
    from workload import bf16_bits_to_f32, round_to_bf16_bits
    q = bf16_bits_to_f32(round_to_bf16_bits(rng.standard_normal((H, N, 64)).astype(np.float32) + 27.0 * u))
    k = bf16_bits_to_f32(round_to_bf16_bits(rng.standard_normal((H, N, 64)).astype(np.float32) + sign * 27.0 * u))
    v = bf16_bits_to_f32(round_to_bf16_bits(rng.standard_normal((H, N, 64)).astype(np.float32)))
    nb = O.num_blocks(N, b)
    mask = _random_mask(H, nb, 0.6, 3)
    idx, cnt = _lists(mask)
    tq, tk, tv = (to_device(x, "bf16") for x in (q, k, v))
    out, lse = B.bsga_sparse_attn(tq, tk, tv, b, idx, cnt, return_lse=True)
    dense, dlse = B.bsga_dense_attn(tq, tk, tv, return_lse=True)
    torch.cuda.synchronize()
    want, want_lse = O.sparse_attention(q, k, v, mask, b, return_lse=True)
    assert abs(np.median(want_lse)) > 80.0  # the case really is out of the fast pass's range
    for got, got_lse, ref, ref_lse in ((out, lse, want, want_lse),
                                       (dense, dlse) + O.dense_attention(q, k, v, return_lse=True)):
        assert torch.isfinite(got.float()).all()
        mx, mean = attn_errors(got, ref)
        assert mx <= 5e-2 and mean <= 5e-3, (mx, mean)
        assert np.abs(got_lse.cpu().numpy() - ref_lse).max() <= 0.25


def test_empty_row_yields_zeros(B):
    H, N, b = 1, 256, 128
    q, k, v = _rand_qkv(H, N, 5, "bf16")
    idx = torch.zeros((H, 2, 2), dtype=torch.int32).cuda()
    cnt = torch.tensor([[0, 1]], dtype=torch.int32).cuda()
    out, lse = B.bsga_sparse_attn(to_device(q, "bf16"), to_device(k, "bf16"), to_device(v, "bf16"), b, idx, cnt,
                                  return_lse=True)
    torch.cuda.synchronize()
    assert (out[0, :128].float() == 0).all() and torch.isinf(lse[0, :128]).all()
    assert torch.isfinite(out.float()).all()


def test_layer_config1_fp32(B):
    """Config 1 end to end: 2 frames, fp32, b=64, tau=0.9, all 16 heads."""
    cfg = CONFIGS[1]
    q, k, v = generate(cfg)
    tq, tk, tv = (to_device(x, cfg.dtype) for x in (q, k, v))
    out, idx, cnt, bits = B.sparse_global_attention(tq, tk, tv, cfg.block, 0.9)
    torch.cuda.synchronize()
    _, _, logits, probs, want_mask = oracle_mask_pipeline(q, k, cfg.block, 0.9, 1.0)
    got_mask = bits_to_mask(bits, cfg.n_blocks)
    unexcused, excused = unexcused_mask_mismatches(got_mask, want_mask, logits, probs, 0.9, 1.0)
    assert unexcused == 0
    want = O.sparse_attention(q, k, v, got_mask, cfg.block)  # same mask on both sides
    mx, mean = attn_errors(out, want)
    print(f"cfg1: kept={got_mask.mean():.4f} excused={excused} max={mx:.2e} mean={mean:.2e}")
    assert mx <= FP32_MAX and mean <= FP32_MEAN, (mx, mean)


@pytest.mark.parametrize("tau", [0.8, 0.9, 0.95, 1.0])
def test_layer_config2_bf16(B, tau):
    """Config 2 end to end: 8 frames, bf16, b=64; tau = 1.0 must equal dense attention."""
    cfg = CONFIGS[2]
    heads = 16 if tau == 0.9 else 4
    q, k, v = generate(cfg, heads=heads)
    tq, tk, tv = (to_device(x, cfg.dtype) for x in (q, k, v))
    out, idx, cnt, bits = B.sparse_global_attention(tq, tk, tv, cfg.block, tau)
    torch.cuda.synchronize()
    _, _, logits, probs, want_mask = oracle_mask_pipeline(q, k, cfg.block, tau, 1.0)
    got_mask = bits_to_mask(bits, cfg.n_blocks)
    unexcused, excused = unexcused_mask_mismatches(got_mask, want_mask, logits, probs, tau, 1.0)
    assert unexcused == 0
    if tau >= 1.0:
        assert got_mask.all()
        want = O.dense_attention(q, k, v)
        dense = B.bsga_dense_attn(tq, tk, tv)
        torch.cuda.synchronize()
        dmx, dmean = attn_errors(dense, want)
        assert dmx <= BF16_MAX and dmean <= BF16_MEAN, (dmx, dmean)
        # the two kernels tile differently (64- vs 128-key tiles) but must agree closely
        assert (out.float() - dense.float()).abs().max().item() <= 4e-3
    else:
        want = O.sparse_attention(q, k, v, got_mask, cfg.block)
    mx, mean = attn_errors(out, want)
    print(f"cfg2 tau={tau}: kept={got_mask.mean():.4f} excused={excused} max={mx:.2e} mean={mean:.2e}")
    assert mx <= BF16_MAX and mean <= BF16_MEAN, (mx, mean)


def test_determinism(B):
    cfg = CONFIGS[2]
    q, k, v = generate(cfg, heads=2, frames=3)
    tq, tk, tv = (to_device(x, cfg.dtype) for x in (q, k, v))
    a = B.sparse_global_attention(tq, tk, tv, cfg.block, 0.9)
    b = B.sparse_global_attention(tq, tk, tv, cfg.block, 0.9)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1][..., :1], b[1][..., :1]) and torch.equal(a[2], b[2])
    assert torch.equal(a[3], b[3])


def test_launch_order_does_not_change_results(B):
    """With a workspace the sparse kernel launches rows much longer than the mean first; without one
    in index order.  Every row must come out bitwise the same either way (the order only decides
    which workgroup computes which row), including empty rows and rows that keep everything."""
    H, N, b = 8, 160 * 128 - 37, 128
    q, k, v = _rand_qkv(H, N, 77, "bf16")
    nb = O.num_blocks(N, b)
    rng = np.random.default_rng(3)
    mask = rng.random((H, nb, nb)) < 0.08
    mask[:, ::17, :] = True            # a few rows keep every block
    mask[:, 5::31, :] = False          # a few rows keep nothing
    idx, cnt = _lists(mask)
    tq, tk, tv = (to_device(x, "bf16") for x in (q, k, v))
    a = B.bsga_sparse_attn(tq, tk, tv, b, idx, cnt, ordered=True)
    c = B.bsga_sparse_attn(tq, tk, tv, b, idx, cnt, ordered=False)
    torch.cuda.synchronize()
    assert torch.equal(a, c)
    assert (a[:, 5 * b:6 * b].float() == 0).all()          # an empty row is zeros
    want = O.sparse_attention(q, k, v, mask, b, q_blocks=[0, 1, 17, nb - 1], heads=[0, 7])
    want[:, 5 * b:6 * b] = np.nan
    assert bf16_bars_ok(a, want)[0], bf16_bars_ok(a, want)


def test_rows_handed_out_at_run_time_do_not_change_results(B):
    """With a workspace, the last eighth of the rows of a large launch is not tied to workgroup
    numbers: workgroups take those rows through a counter (an XCD that runs faster takes more).
    Which workgroup computes a row must not matter: dense attention with and without the workspace
    is bitwise the same, call after call (the counter is cleared by every call), and so is the
    block-sparse kernel on a keep-all list."""
    H, N, b = 10, 128 * 128 + 77, 128             # 1290 rows: above the 1024 that switch the hand-out on
    q, k, v = _rand_qkv(H, N, 78, "bf16")
    tq, tk, tv = (to_device(x, "bf16") for x in (q, k, v))
    plain = B.bsga_dense_attn(tq, tk, tv, balanced=False)
    for _ in range(3):
        assert torch.equal(B.bsga_dense_attn(tq, tk, tv), plain)
    nb = O.num_blocks(N, b)
    idx, cnt = _lists(np.ones((H, nb, nb), dtype=bool))
    for _ in range(2):
        assert torch.equal(B.bsga_sparse_attn(tq, tk, tv, b, idx, cnt), plain)
    want = O.sparse_attention(q, k, v, np.ones((H, nb, nb), dtype=bool), b, q_blocks=[0, nb - 2, nb - 1], heads=[0, 9])
    assert bf16_bars_ok(plain, want)[0], bf16_bars_ok(plain, want)
