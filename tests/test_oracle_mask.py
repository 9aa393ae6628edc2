"""Pins for the oracle's mask predictor (pooling, block scores, block softmax,
selection) against facts fixed by the paper's definitions (Sec. 4.1) and by
arithmetic, not by the oracle itself."""
import math

import numpy as np
import pytest

from oracle import bsga_oracle as O


def _rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# ---- pooling + scores --------------------------------------------------------------
@pytest.mark.parametrize("N,b", [(24, 4), (23, 4), (130, 64), (7, 8)])
def test_pooled_score_is_mean_of_explicit_block_scores(N, b):
    """Bilinearity: P(Q)_I . P(K)_J equals the mean of q_i . k_j over the block
    pair, ragged tail included (mean over valid tokens)."""
    H, d = 2, 5
    q, k = _rand((H, N, d), 1), _rand((H, N, d), 2)
    S = O.block_logits(O.pool_blocks(q, b), O.pool_blocks(k, b), 1.0)
    nb = O.num_blocks(N, b)
    assert S.shape == (H, nb, nb)
    for h in range(H):
        full = q[h] @ k[h].T
        for I in range(nb):
            for J in range(nb):
                blk = full[I * b:min((I + 1) * b, N), J * b:min((J + 1) * b, N)]
                assert abs(S[h, I, J] - blk.mean()) < 1e-12


def test_pool_hand_values_and_tail():
    x = np.arange(10, dtype=np.float64).reshape(1, 5, 2)  # tokens (0,1),(2,3),(4,5),(6,7),(8,9)
    p = O.pool_blocks(x, 2)
    assert p.shape == (1, 3, 2)
    np.testing.assert_array_equal(p[0], [[1.0, 2.0], [5.0, 6.0], [8.0, 9.0]])  # tail = its single token


def test_score_scale_is_applied_once():
    qp, kp = _rand((1, 3, 4), 3), _rand((1, 2, 4), 4)
    a = O.block_logits(qp, kp, 1.0)
    b = O.block_logits(qp, kp, 0.125)
    np.testing.assert_allclose(b, 0.125 * a, rtol=1e-15)
    assert a.shape == (1, 3, 2)
    assert abs(a[0, 2, 1] - float(qp[0, 2] @ kp[0, 1])) < 1e-14  # not transposed


# ---- block softmax -----------------------------------------------------------------
def test_block_softmax_rows():
    L = 5.0 * _rand((2, 7, 11), 5)
    P = O.block_softmax(L)
    np.testing.assert_allclose(P.sum(-1), 1.0, atol=1e-12)
    assert (P > 0).all()
    np.testing.assert_allclose(O.block_softmax(L + 123.0), P, atol=1e-12)  # shift invariance
    # closed form: logits (0, ln 3) -> (1/4, 3/4)
    np.testing.assert_allclose(O.block_softmax(np.array([[[0.0, math.log(3.0)]]]))[0, 0], [0.25, 0.75], atol=1e-15)
    # huge logits must not overflow
    assert np.isfinite(O.block_softmax(np.array([[[1000.0, 999.0]]]))).all()


# ---- selection ---------------------------------------------------------------------
def test_topk_floor_arithmetic():
    assert O.topk_floor(43, 0.75) == 10      # floor(10.75)
    assert O.topk_floor(1074, 0.5) == 537
    assert O.topk_floor(1074, 0.9) == 107    # floor(107.4)
    assert O.topk_floor(43, 1.0) == 0
    assert O.topk_floor(43, 0.0) == 43


def test_hand_worked_row():
    """p = (.1,.4,.2,.3): ranking 1,3,2,0; cumulative .4,.7,.9,1.0."""
    p = np.array([0.1, 0.4, 0.2, 0.3])
    s = O.select_row(p, 0.65, 1.0)
    assert list(s.order) == [1, 3, 2, 0]
    assert s.n_cdf == 2 and s.n_keep == 2
    assert O.select_row(p, 0.69, 1.0).n_keep == 2       # .4 + .3 covers .69 ...
    assert O.select_row(p, 0.71, 1.0).n_keep == 3
    assert O.select_row(p, 0.05, 1.0).n_keep == 1
    assert O.select_row(p, 0.0, 1.0).n_keep == 1        # never an empty row
    assert O.select_row(p, 1.0, 1.0).n_keep == 4        # tau >= 1 keeps everything
    assert O.select_row(p, 0.05, 0.5).n_keep == 2       # top-k floor: floor(4*0.5)=2 beats n_cdf=1
    assert O.select_row(p, 0.95, 0.5).n_keep == 4       # CDF beats the floor
    m = O.select_blocks(p[None, None, :], 0.65, 1.0)
    assert m.tolist() == [[[False, True, False, True]]]


def test_cdf_boundary_is_inclusive():
    p = np.array([0.5, 0.25, 0.25])  # exact in binary
    assert O.select_row(p, 0.5, 1.0).n_keep == 1   # c_1 = 0.5 >= tau
    assert O.select_row(p, 0.75, 1.0).n_keep == 2
    assert O.select_row(p, 0.7500001, 1.0).n_keep == 3


def test_uniform_row_closed_form_and_tie_break():
    """All keys equal -> uniform distribution -> n = ceil(tau * NB), lowest indices first."""
    H, nbq, nbk, d = 1, 3, 37, 8
    qp = _rand((H, nbq, d), 6)
    kp = np.tile(_rand((1, 1, d), 7), (H, nbk, 1))
    P = O.block_softmax(O.block_logits(qp, kp, 1.0))
    for tau in (0.3, 0.77, 0.9):
        n = math.ceil(tau * nbk)
        assert abs(tau * nbk - round(tau * nbk)) > 1e-3
        m = O.select_blocks(P, tau, 1.0)
        assert (m.sum(-1) == n).all()
        assert m[:, :, :n].all() and not m[:, :, n:].any()


def test_planted_one_hot():
    """Orthogonal scaled codes -> near one-hot distribution -> only the planted column is kept."""
    nb, d = 8, 8
    codes = 12.0 * np.eye(d)[None]
    perm = np.array([3, 1, 7, 0, 2, 6, 5, 4])
    qp = codes[:, perm, :]
    P = O.block_softmax(O.block_logits(qp, codes, 1.0))
    m = O.select_blocks(P, 0.9, 1.0)
    assert (m.sum(-1) == 1).all()
    assert (np.argmax(m[0], axis=1) == perm).all()


def _random_probs(seed, H=2, nbq=6, nbk=29, sharp=3.0):
    return O.block_softmax(sharp * _rand((H, nbq, nbk), seed))


@pytest.mark.parametrize("tau,rho", [(0.5, 1.0), (0.9, 1.0), (0.9, 0.6), (0.2, 0.8)])
def test_selection_invariants(tau, rho):
    P = _random_probs(11)
    m = O.select_blocks(P, tau, rho)
    k = O.topk_floor(P.shape[-1], rho)
    for h in range(P.shape[0]):
        for I in range(P.shape[1]):
            p, kept = P[h, I], m[h, I]
            n = int(kept.sum())
            assert n >= max(k, 1)
            assert p[kept].min() >= p[~kept].max() if n < p.size else True   # top-ranked set
            assert p[kept].sum() >= tau - 1e-12                                # coverage
            if n > max(k, 1):                                                  # CDF decided: minimal prefix
                assert p[kept].sum() - p[kept].min() < tau


def test_nesting_in_tau_and_rho():
    P = _random_probs(12)
    prev = None
    for tau in (0.1, 0.5, 0.8, 0.95, 1.0):
        m = O.select_blocks(P, tau, 1.0)
        if prev is not None:
            assert (m | ~prev).all()
        prev = m
    assert prev.all()
    prev = None
    for rho in (1.0, 0.9, 0.5, 0.1, 0.0):
        m = O.select_blocks(P, 0.3, rho)
        if prev is not None:
            assert (m | ~prev).all()
        prev = m
    assert prev.all()


def test_column_permutation_equivariance():
    P = _random_probs(13)
    perm = np.random.default_rng(0).permutation(P.shape[-1])
    m = O.select_blocks(P, 0.8, 0.9)
    mp = O.select_blocks(P[:, :, perm], 0.8, 0.9)
    assert (mp == m[:, :, perm]).all()


def test_force_rows_and_columns():
    P = _random_probs(14)
    fq = np.zeros(P.shape[1], np.uint8); fq[2] = 1
    fk = np.zeros(P.shape[2], np.uint8); fk[[0, 5]] = 1
    base = O.select_blocks(P, 0.5, 1.0)
    m = O.select_blocks(P, 0.5, 1.0, fq, fk)
    assert m[:, 2, :].all() and m[:, :, 0].all() and m[:, :, 5].all()
    rest = np.ones_like(m); rest[:, 2, :] = False; rest[:, :, [0, 5]] = False
    assert (m[rest] == base[rest]).all()


def test_index_lists_and_bits_roundtrip():
    P = _random_probs(15, nbk=70)
    m = O.select_blocks(P, 0.6, 1.0)
    idx, cnt = O.mask_to_index_lists(m)
    bits = O.mask_to_bits(m)
    assert bits.shape[-1] == 3
    for h in range(m.shape[0]):
        for I in range(m.shape[1]):
            js = idx[h, I, :cnt[h, I]]
            assert (np.diff(js) > 0).all()
            assert set(js.tolist()) == set(np.flatnonzero(m[h, I]).tolist())
            assert (idx[h, I, cnt[h, I]:] == -1).all()
            for J in range(70):
                assert bool((bits[h, I, J // 32] >> np.uint32(J % 32)) & np.uint32(1)) == bool(m[h, I, J])


@pytest.mark.parametrize("scale", [1.0, None])
def test_predict_mask_matches_manual_chain_on_tiny_case(scale):
    """Brute force of steps 1-4 with python loops on a tiny ragged case; scale None is the
    default block-score scale 1/sqrt(d_h) (here 1/sqrt(3), with inputs large enough that the two
    scales select different blocks)."""
    H, N, d, b = 1, 11, 3, 4
    q, k = 2.0 * _rand((H, N, d), 20), 2.0 * _rand((H, N, d), 21)
    tau = 0.6
    m = O.predict_mask(q, k, b, tau, 1.0, score_scale=1.0) if scale is not None else O.predict_mask(q, k, b, tau, 1.0)
    if scale is None:
        assert (m != O.predict_mask(q, k, b, tau, 1.0, score_scale=1.0)).any()  # the case tells the scales apart
    factor = 1.0 if scale is not None else 1.0 / math.sqrt(d)
    nb = 3
    blocks = [range(0, 4), range(4, 8), range(8, 11)]
    for I in range(nb):
        s = []
        for J in range(nb):
            tot = 0.0
            for i in blocks[I]:
                for j in blocks[J]:
                    tot += float(np.dot(q[0, i], k[0, j]))
            s.append(factor * tot / (len(blocks[I]) * len(blocks[J])))
        e = [math.exp(x - max(s)) for x in s]
        p = [x / sum(e) for x in e]
        order = sorted(range(nb), key=lambda j: (-p[j], j))
        acc, keep = 0.0, set()
        for j in order:
            keep.add(j); acc += p[j]
            if acc >= tau:
                break
        assert set(np.flatnonzero(m[0, I]).tolist()) == keep


# ---- two separately blocked parts (Sec. 4.2) ----------------------------------------------------
def test_block_ranges_and_split_pooling():
    """Blocks never cross n_first; each part ends in its own short block; pooled values are plain
    means of exactly those tokens."""
    assert O.block_ranges(11, 4) == [(0, 4), (4, 8), (8, 11)]
    assert O.block_ranges(11, 4, 6) == [(0, 4), (4, 6), (6, 10), (10, 11)]
    assert O.block_ranges(11, 4, 11) == O.block_ranges(11, 4) == O.block_ranges(11, 4, 0)
    assert O.block_ranges(8, 4, 4) == [(0, 4), (4, 8)]
    x = np.arange(22, dtype=np.float64).reshape(1, 11, 2)
    p = O.pool_blocks(x, 4, n_first=6)
    assert p.shape == (1, 4, 2)
    np.testing.assert_array_equal(p[0, :, 0], [(0 + 2 + 4 + 6) / 4, (8 + 10) / 2, (12 + 14 + 16 + 18) / 4, 20.0])
