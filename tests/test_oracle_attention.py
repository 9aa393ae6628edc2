"""Pins for the oracle's attention functions (Eqs. (1) and (2)): brute force at
token level, a library routine, closed forms and bounds that follow from the
definition of softmax attention."""
import math

import numpy as np
import pytest
import torch

from oracle import bsga_oracle as O


def _rand(shape, seed, scale=1.0):
    return scale * np.random.default_rng(seed).standard_normal(shape)


def _token_level_bruteforce(q, k, v, mask, b):
    """Expand the block mask to an N x N token matrix and evaluate the masked
    softmax row by row with python loops."""
    H, N, d = q.shape
    out = np.zeros((H, N, d))
    for h in range(H):
        for i in range(N):
            w = []
            for j in range(N):
                if mask[h, i // b, j // b]:
                    w.append((j, math.exp(sum(q[h, i, t] * k[h, j, t] for t in range(d)) / math.sqrt(d))))
            z = sum(x for _, x in w)
            for j, x in w:
                for t in range(d):
                    out[h, i, t] += (x / z) * v[h, j, t]
    return out


@pytest.mark.parametrize("N", [24, 22])
def test_sparse_attention_vs_token_level_bruteforce(N):
    H, d, b = 2, 4, 4
    q, k, v = _rand((H, N, d), 1), _rand((H, N, d), 2), _rand((H, N, d), 3)
    nb = O.num_blocks(N, b)
    mask = np.random.default_rng(4).random((H, nb, nb)) < 0.4
    mask[:, np.arange(nb), np.arange(nb)] = True  # no empty rows
    got = O.sparse_attention(q, k, v, mask, b)
    np.testing.assert_allclose(got, _token_level_bruteforce(q, k, v, mask, b), atol=1e-12)


def test_keep_all_equals_dense_function():
    H, N, d, b = 2, 150, 8, 64
    q, k, v = _rand((H, N, d), 5), _rand((H, N, d), 6), _rand((H, N, d), 7)
    nb = O.num_blocks(N, b)
    o_s, l_s = O.sparse_attention(q, k, v, np.ones((H, nb, nb), bool), b, return_lse=True)
    o_d, l_d = O.dense_attention(q, k, v, row_chunk=64, return_lse=True)
    np.testing.assert_allclose(o_s, o_d, atol=1e-12)
    np.testing.assert_allclose(l_s, l_d, atol=1e-12)


def test_dense_vs_library_routine():
    H, N, d = 3, 97, 16
    q, k, v = _rand((H, N, d), 8), _rand((H, N, d), 9), _rand((H, N, d), 10)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None])[0].numpy()
    np.testing.assert_allclose(O.dense_attention(q, k, v), ref, atol=1e-12)


def test_closed_form_two_keys_pins_the_scale():
    """d_h = 4, q = (2,0,0,0), k_0 = 0, k_1 = (ln 3,0,0,0): logits (0, 2 ln3 / sqrt 4 = ln 3)
    -> weights (1/4, 3/4)."""
    q = np.zeros((1, 2, 4)); q[0, :, 0] = 2.0
    k = np.zeros((1, 2, 4)); k[0, 1, 0] = math.log(3.0)
    v = np.array([[[1.0, 0.0, 0.0, 8.0], [0.0, 1.0, 0.0, -8.0]]])
    o, lse = O.dense_attention(q, k, v, return_lse=True)
    np.testing.assert_allclose(o[0, 0], [0.25, 0.75, 0.0, -4.0], atol=1e-14)
    np.testing.assert_allclose(lse[0], math.log(4.0), atol=1e-14)
    o2 = O.sparse_attention(q, k, v, np.ones((1, 1, 1), bool), 2)
    np.testing.assert_allclose(o2[0, 1], [0.25, 0.75, 0.0, -4.0], atol=1e-14)


def test_masked_entries_are_excluded_not_zeroed():
    """If a masked logit were set to 0 it would still get weight; with exclusion
    a row that keeps one single-token block returns that token's value exactly."""
    H, N, d, b = 1, 4, 2, 1
    q, k, v = _rand((H, N, d), 11), _rand((H, N, d), 12), _rand((H, N, d), 13)
    mask = np.eye(4, dtype=bool)[None][:, :, ::-1]  # row i keeps only key 3-i
    o = O.sparse_attention(q, k, v, mask, b)
    np.testing.assert_allclose(o[0], v[0, ::-1], atol=1e-15)


def test_equal_keys_give_mean_of_values():
    H, N, d = 1, 10, 4
    q, v = _rand((H, N, d), 14), _rand((H, N, d), 15)
    k = np.tile(_rand((1, 1, d), 16), (1, N, 1))
    np.testing.assert_allclose(O.dense_attention(q, k, v)[0], np.tile(v[0].mean(0), (N, 1)), atol=1e-13)


def test_convexity_and_kept_block_permutation():
    H, N, d, b = 1, 40, 4, 8
    q, k, v = _rand((H, N, d), 17, 2.0), _rand((H, N, d), 18, 2.0), _rand((H, N, d), 19)
    nb = 5
    mask = np.zeros((H, nb, nb), bool); mask[:, :, [0, 2, 3]] = True
    o = O.sparse_attention(q, k, v, mask, b)
    kept_tokens = np.r_[0:8, 16:32]
    assert (o[0] <= v[0, kept_tokens].max(0) + 1e-12).all() and (o[0] >= v[0, kept_tokens].min(0) - 1e-12).all()
    # swap key blocks 0 and 3 (with their values) and the mask columns: output unchanged
    perm = np.r_[24:32, 8:16, 16:24, 0:8, 32:40]
    o2 = O.sparse_attention(q, k[:, perm], v[:, perm], mask[:, :, [3, 1, 2, 0, 4]], b)
    np.testing.assert_allclose(o2, o, atol=1e-12)
    # dropped block's content is irrelevant
    k3, v3 = k.copy(), v.copy(); k3[:, 8:16] += 100.0; v3[:, 32:40] = 1e6
    np.testing.assert_allclose(O.sparse_attention(q, k3, v3, mask, b), o, atol=1e-12)


def test_dropped_mass_error_bound():
    """|o_sparse - o_dense|_inf <= 2 * delta_i * max|v| with delta_i the dense
    attention mass of row i on dropped keys."""
    H, N, d, b = 2, 96, 8, 8
    q, k, v = _rand((H, N, d), 20, 1.5), _rand((H, N, d), 21, 1.5), _rand((H, N, d), 22)
    mask = O.predict_mask(q, k, b, 0.7, 1.0)
    o_s = O.sparse_attention(q, k, v, mask, b)
    o_d = O.dense_attention(q, k, v)
    tok_mask = np.repeat(np.repeat(mask, b, axis=1), b, axis=2)[:, :N, :N]
    for h in range(H):
        L = q[h] @ k[h].T / math.sqrt(d)
        Pd = np.exp(L - L.max(1, keepdims=True)); Pd /= Pd.sum(1, keepdims=True)
        delta = (Pd * ~tok_mask[h]).sum(1)
        err = np.abs(o_s[h] - o_d[h]).max(1)
        assert (err <= 2 * delta * np.abs(v[h]).max() + 1e-12).all()
    assert not mask.all()  # the case really drops something


def test_ragged_tail_and_sampled_blocks():
    H, N, d, b = 1, 21, 4, 8
    q, k, v = _rand((H, N, d), 23), _rand((H, N, d), 24), _rand((H, N, d), 25)
    mask = np.array([[[1, 0, 1], [0, 1, 1], [1, 1, 0]]], bool)
    full = O.sparse_attention(q, k, v, mask, b)
    np.testing.assert_allclose(full, _token_level_bruteforce(q, k, v, mask, b), atol=1e-12)
    part = O.sparse_attention(q, k, v, mask, b, q_blocks=[2])
    assert np.isnan(part[0, :16]).all()
    np.testing.assert_array_equal(part[0, 16:], full[0, 16:])


def test_whole_layer_tau_one_is_dense():
    H, N, d, b = 2, 100, 8, 16
    q, k, v = _rand((H, N, d), 26), _rand((H, N, d), 27), _rand((H, N, d), 28)
    o, m = O.sparse_global_attention(q, k, v, b, 1.0, 1.0)
    assert m.all()
    np.testing.assert_allclose(o, O.dense_attention(q, k, v), atol=1e-12)


# --------------------------------------------------------------------------- separate q / k block sizes
def test_asymmetric_blocks_token_level_brute_force():
    """Query blocks of 8, key blocks of 4: every row against a literal masked softmax."""
    rng = np.random.default_rng(11)
    H, N, d, bq, bk = 2, 27, 4, 8, 4
    q, k, v = (rng.standard_normal((H, N, d)) for _ in range(3))
    q *= 2.0
    mask = O.predict_mask(q, k, bq, 0.6, 1.0, b_k=bk)
    assert mask.shape == (H, 4, 7) and not mask.all()
    out = O.sparse_attention(q, k, v, mask, bq, b_k=bk)
    for h in range(H):
        allowed = np.zeros((N, N), dtype=bool)
        for i in range(N):
            for j in range(N):
                allowed[i, j] = mask[h, i // bq, j // bk]
        logits = (q[h] @ k[h].T) / np.sqrt(d)
        logits[~allowed] = -np.inf
        w = np.exp(logits - logits.max(axis=1, keepdims=True))
        np.testing.assert_allclose(out[h], (w / w.sum(axis=1, keepdims=True)) @ v[h], rtol=0, atol=1e-12)


def test_asymmetric_blocks_keep_all_is_dense_and_pooling_is_per_side():
    rng = np.random.default_rng(12)
    H, N, d = 1, 40, 8
    q, k, v = (rng.standard_normal((H, N, d)) for _ in range(3))
    full = np.ones((H, 3, 5), dtype=bool)
    np.testing.assert_allclose(O.sparse_attention(q, k, v, full, 16, b_k=8), O.dense_attention(q, k, v), rtol=0, atol=1e-12)
    # the block scores are the means of the explicit token scores of each (16 x 8) rectangle
    logits = O.block_logits(O.pool_blocks(q, 16), O.pool_blocks(k, 8), 1.0)
    s = q[0] @ k[0].T
    for I in range(3):
        for J in range(5):
            want = s[I * 16:min((I + 1) * 16, N), J * 8:(J + 1) * 8].mean()
            assert abs(logits[0, I, J] - want) < 1e-12


# --------------------------------------------------------------------------- two separately blocked parts
def test_split_blocks_token_level_brute_force():
    """Sec. 4.2 blocking (tokens [0, n_first) and [n_first, N) cut into blocks separately), also
    with separate query / key block sizes: every row against a literal masked softmax built from
    an explicit token -> block map."""
    rng = np.random.default_rng(13)
    H, N, d, n_first = 2, 29, 4, 13
    q, k, v = (rng.standard_normal((H, N, d)) for _ in range(3))
    for bq, bk in ((4, 4), (8, 4)):
        def block_of(t, b):  # written out, not taken from the oracle
            return t // b if t < n_first else -(-n_first // b) + (t - n_first) // b
        nbq = -(-n_first // bq) + -(-(N - n_first) // bq)
        nbk = -(-n_first // bk) + -(-(N - n_first) // bk)
        mask = rng.random((H, nbq, nbk)) < 0.5
        mask[:, :, 0] = True
        out, lse = O.sparse_attention(q, k, v, mask, bq, b_k=bk, n_first=n_first, return_lse=True)
        for h in range(H):
            allowed = np.array([[mask[h, block_of(i, bq), block_of(j, bk)] for j in range(N)] for i in range(N)])
            logits = (q[h] @ k[h].T) / np.sqrt(d)
            logits[~allowed] = -np.inf
            w = np.exp(logits - logits.max(axis=1, keepdims=True))
            np.testing.assert_allclose(out[h], (w / w.sum(axis=1, keepdims=True)) @ v[h], rtol=0, atol=1e-12)
            np.testing.assert_allclose(lse[h], np.log(np.exp(logits).sum(axis=1)), rtol=0, atol=1e-12)


def test_split_with_everything_kept_is_dense_and_matches_special_token_statement():
    rng = np.random.default_rng(14)
    H, N, d, b, n_first = 1, 37, 8, 8, 27
    q, k, v = (rng.standard_normal((H, N, d)) for _ in range(3))
    nb = len(O.block_ranges(N, b, n_first))
    np.testing.assert_allclose(O.sparse_attention(q, k, v, np.ones((H, nb, nb), bool), b, n_first=n_first),
                               O.dense_attention(q, k, v), rtol=0, atol=1e-12)
    # patch tokens first, special tokens last: the split blocking with dense special rows / columns
    # is the special-token statement of Sec. 4.2
    patch_idx, special_idx = np.arange(n_first), np.arange(n_first, N)
    want, pmask = O.special_token_attention(2.0 * q, k, v, patch_idx, special_idx, b, 0.6, 1.0)
    npb = pmask.shape[-1]
    mask = np.ones((H, nb, nb), bool)
    mask[:, :npb, :npb] = pmask
    assert not pmask.all()
    np.testing.assert_allclose(O.sparse_attention(2.0 * q, k, v, mask, b, n_first=n_first), want, rtol=0, atol=1e-12)
