"""Pins for the oracle's special-token path (Sec. 4.2): block map on patch tokens only, everything
that touches a special token dense."""
import numpy as np
import pytest

from oracle import bsga_oracle as O


def _tokens(frames, per_frame, n_special):
    """Frame-interleaved layout: each frame starts with n_special special tokens."""
    idx = np.arange(frames * per_frame)
    special = (idx % per_frame) < n_special
    return np.flatnonzero(~special), np.flatnonzero(special)


def _rand(H, N, d, seed):
    rng = np.random.default_rng(seed)
    return tuple(rng.standard_normal((H, N, d)) for _ in range(3))


def test_token_level_brute_force():
    """Every output row against a literal masked softmax over an explicit N x N pair mask."""
    frames, per_frame, ns, b, d, H = 3, 11, 2, 4, 4, 2
    patch, special = _tokens(frames, per_frame, ns)
    q, k, v = _rand(H, frames * per_frame, d, 1)
    q *= 2.0
    out, mask = O.special_token_attention(q, k, v, patch, special, b, 0.6, 1.0)
    N = q.shape[1]
    assert not mask.all(), "the case must actually drop blocks"
    block_of = np.full(N, -1)
    block_of[patch] = np.arange(patch.size) // b  # block of a patch token in the patch-only sequence
    for h in range(H):
        allowed = np.zeros((N, N), dtype=bool)
        allowed[special, :] = True
        allowed[:, special] = True
        for i in patch:
            for j in patch:
                allowed[i, j] = mask[h, block_of[i], block_of[j]]
        logits = (q[h] @ k[h].T) / np.sqrt(d)
        logits[~allowed] = -np.inf
        w = np.exp(logits - logits.max(axis=1, keepdims=True))
        want = (w / w.sum(axis=1, keepdims=True)) @ v[h]
        np.testing.assert_allclose(out[h], want, rtol=0, atol=1e-12)


def test_special_rows_are_dense_rows_and_tau_one_is_dense():
    frames, per_frame, ns, b = 4, 13, 3, 4
    patch, special = _tokens(frames, per_frame, ns)
    q, k, v = _rand(2, frames * per_frame, 8, 2)
    dense = O.dense_attention(q, k, v)
    out, _ = O.special_token_attention(q, k, v, patch, special, b, 0.5, 1.0)
    np.testing.assert_allclose(out[:, special], dense[:, special], rtol=0, atol=1e-12)
    assert np.abs(out[:, patch] - dense[:, patch]).max() > 1e-6  # patch rows really are sparse
    full, mask = O.special_token_attention(q, k, v, patch, special, b, 1.0, 1.0)
    assert mask.all()
    np.testing.assert_allclose(full, dense, rtol=0, atol=1e-12)


def test_without_special_tokens_it_is_the_plain_path():
    q, k, v = _rand(2, 50, 8, 3)
    out, mask = O.special_token_attention(q, k, v, np.arange(50), np.arange(0), 8, 0.7, 0.9)
    want, want_mask = O.sparse_global_attention(q, k, v, 8, 0.7, 0.9)
    assert (mask == want_mask).all()
    np.testing.assert_allclose(out, want, rtol=0, atol=1e-13)


def test_patch_order_defines_the_blocks():
    """The block map is pooled over consecutive entries of patch_idx: moving the special tokens
    elsewhere in the sequence does not change any output."""
    frames, per_frame, ns, b = 3, 10, 2, 4
    patch, special = _tokens(frames, per_frame, ns)
    q, k, v = _rand(1, frames * per_frame, 4, 4)
    out, mask = O.special_token_attention(q, k, v, patch, special, b, 0.6, 1.0)
    order = np.concatenate([patch, special])  # specials moved to the end
    q2, k2, v2 = q[:, order], k[:, order], v[:, order]
    out2, mask2 = O.special_token_attention(q2, k2, v2, np.arange(patch.size),
                                            np.arange(patch.size, order.size), b, 0.6, 1.0)
    assert (mask == mask2).all()
    np.testing.assert_allclose(out2, out[:, order], rtol=0, atol=1e-12)


def test_unranked_columns():
    rng = np.random.default_rng(5)
    H, nbq, nbk = 2, 6, 10
    logits = rng.standard_normal((H, nbq, nbk)) * 2.0
    none = np.zeros(nbk, dtype=bool)
    plain = O.select_blocks(O.block_softmax(logits), 0.6, 1.0)
    assert (O.select_blocks_unranked_columns(logits, 0.6, 1.0, none) == plain).all()
    dense_k = none.copy()
    dense_k[[2, 7]] = True
    m = O.select_blocks_unranked_columns(logits, 0.6, 1.0, dense_k)
    assert m[:, :, dense_k].all()
    # the logits of unranked columns are irrelevant
    other = logits.copy()
    other[:, :, dense_k] = 50.0
    assert (O.select_blocks_unranked_columns(other, 0.6, 1.0, dense_k) == m).all()
    # the kept ranked columns hold >= tau of the mass of the ranked columns, minimally
    ranked = ~dense_k
    p = np.exp(logits[:, :, ranked])
    p /= p.sum(-1, keepdims=True)
    kept = m[:, :, ranked]
    mass = (p * kept).sum(-1)
    assert (mass >= 0.6 - 1e-12).all()
    smallest_kept = np.where(kept, p, np.inf).min(-1)
    assert ((mass - smallest_kept < 0.6) | (kept.sum(-1) == 1)).all()
    # top-k floor counts ranked blocks only: B = 8, rho = 0.5 -> 4 ranked blocks + the 2 unranked
    topk = O.select_blocks_unranked_columns(logits, 0.0, 0.5, dense_k)
    assert (topk.sum(-1) == 4 + 2).all()
    # dense query rows
    dq = np.zeros(nbq, dtype=bool)
    dq[1] = True
    assert O.select_blocks_unranked_columns(logits, 0.3, 1.0, dense_k, dq)[:, 1].all()
