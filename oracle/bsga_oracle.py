"""CPU oracle for block-sparse global attention.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what the hot path computes, written
from the paper (Sec. 4.1, Eqs. (1)-(2), paragraphs "Predicting Block Masks"
and "Selecting Blocks"; Sec. 4.2 for the special-token hooks).  It shares no
code with the HIP path and must never be imported by the product package:
only the tests, the smoke check and the benchmark's CPU-baseline leg use it.

Steps, in the paper's order:
  1. pool_blocks      P^b(Q), P^b(K): block average pooling, block size b.
  2. block_logits     S = P^b(Q) P^b(K)^T, times a score scale.
  3. block_softmax    row softmax of S -> a distribution over key blocks.
  4. select_blocks    CDF threshold tau united with a top-k floor
                      k = floor(B (1 - rho)) -> binary block mask M.
  5. sparse_attention Eq. (2): softmax attention restricted to kept blocks.
  6. dense_attention  Eq. (1).
  7. special_token_attention  Sec. 4.2: the block map is predicted and applied
                      on patch tokens only; special tokens attend and are
                      attended densely.

Readings taken where the paper is silent or ambiguous (each is restated at the
function that uses it):
  * Eq. (2) multiplies logits by M; read literally a masked entry would get
    logit 0 and still take part in the softmax.  The text says only the kept
    entries are computed, so masked entries are excluded (logit -inf).
  * The block logits carry a caller-chosen scale (default 1/sqrt(d_h), since
    the pooled map is described as a low-resolution attention map; 1.0 is the
    literal formula).
  * B is the number of key blocks of one query-block row.
  * The two criteria share one ranking; the kept set is the top
    max(n_cdf, k, 1) blocks of it.  n_cdf is the shortest prefix whose mass is
    >= tau; tau >= 1 keeps every block.
  * Equal probabilities rank lower key-block index first.
  * A ragged last block is averaged over its valid tokens only; the block
    softmax is not weighted by block size.

Pins (tests/test_oracle_*.py): bilinearity of pooled scores, softmax row sums,
selection minimality/nesting/closed forms, a token-level brute force of the
masked softmax, keep-all == dense, dense == a library attention routine, a
closed-form two-key example, and the dropped-mass error bound; for Sec. 4.2
a token-level brute force with an explicit pair mask, special rows == dense
rows, no special tokens == the plain path, and everything-kept == dense.
Parity unpinned: the paper's task-accuracy claims (they need datasets and
trained weights).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Iterable, Optional, Sequence

import numpy as np


def num_blocks(n_tokens: int, b: int) -> int:
    return (n_tokens + b - 1) // b


def block_ranges(n_tokens: int, b: int, n_first: Optional[int] = None):
    """Token ranges [lo, hi) of the blocks of size b.  With n_first given, tokens [0, n_first) and
    [n_first, n_tokens) are cut into blocks separately, so no block holds tokens of both parts
    (Sec. 4.2: patch tokens and special tokens are kept apart); the last block of each part may be
    short.  Without it: consecutive blocks, the last one possibly short."""
    parts = [(0, n_tokens)] if n_first is None else [(0, n_first), (n_first, n_tokens)]
    out = []
    for lo, hi in parts:
        for s in range(lo, hi, b):
            out.append((s, min(s + b, hi)))
    return out


# --------------------------------------------------------------------------- step 1
def pool_blocks(x: np.ndarray, b: int, n_first: Optional[int] = None) -> np.ndarray:
    """Block average pooling P^b(x) (Sec. 4.1, "Predicting Block Masks").

    x: [H, N, d].  Returns [H, number of blocks, d] in fp64.  Block I covers tokens
    I*b .. min((I+1)*b, N)-1 (or, with n_first, the ranges of block_ranges) and is averaged over
    exactly those tokens.
    """
    x = np.asarray(x, dtype=np.float64)
    H, N, d = x.shape
    ranges = block_ranges(N, b, n_first)
    out = np.empty((H, len(ranges), d), dtype=np.float64)
    for I, (lo, hi) in enumerate(ranges):
        out[:, I, :] = x[:, lo:hi, :].sum(axis=1) / float(hi - lo)
    return out


# --------------------------------------------------------------------------- step 2
def block_logits(q_pool: np.ndarray, k_pool: np.ndarray, score_scale: float) -> np.ndarray:
    """score_scale * P^b(Q) P^b(K)^T per head: [H, NBq, NBk]."""
    q_pool = np.asarray(q_pool, dtype=np.float64)
    k_pool = np.asarray(k_pool, dtype=np.float64)
    return score_scale * np.einsum("hid,hjd->hij", q_pool, k_pool)


# --------------------------------------------------------------------------- step 3
def block_softmax(logits: np.ndarray) -> np.ndarray:
    """Row softmax over key blocks (last axis), max-subtracted."""
    z = logits - logits.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


# --------------------------------------------------------------------------- step 4
def topk_floor(nb_k: int, rho: float) -> int:
    """k = floor(B (1 - rho)), B = number of key blocks in a row (Sec. 4.1,
    "Selecting Blocks"); evaluated in binary64 exactly as written."""
    return int(math.floor(nb_k * (1.0 - rho)))


@dataclass
class RowSelection:
    order: np.ndarray  # key-block indices, best first
    cum: np.ndarray  # cumulative probability in that order
    n_cdf: int
    n_keep: int


def select_row(p: np.ndarray, tau: float, rho: float) -> RowSelection:
    """Rank one row's key blocks and decide how many to keep.

    order: descending probability, equal values by ascending block index.
    n_cdf: smallest r with p[order[0]] + ... + p[order[r-1]] >= tau (summed in
           rank order); all blocks when tau >= 1 or the sum never reaches tau.
    kept:  the first max(n_cdf, k, 1) of the ranking, capped at the row length.
    """
    nb_k = p.shape[0]
    order = np.argsort(-p, kind="stable")
    cum = np.cumsum(p[order])
    if tau >= 1.0:
        n_cdf = nb_k
    else:
        reached = np.flatnonzero(cum >= tau)
        n_cdf = int(reached[0]) + 1 if reached.size else nb_k
    n_keep = min(nb_k, max(n_cdf, topk_floor(nb_k, rho), 1))
    return RowSelection(order, cum, n_cdf, n_keep)


def select_blocks(
    probs: np.ndarray,
    tau: float,
    rho: float,
    force_q: Optional[np.ndarray] = None,
    force_k: Optional[np.ndarray] = None,
) -> np.ndarray:
    """Binary block mask M [H, NBq, NBk] from the block distributions.

    force_q[I] != 0 keeps the whole row I, force_k[J] != 0 keeps column J in
    every row (Sec. 4.2: interactions that involve special tokens stay dense).
    """
    H, nbq, nbk = probs.shape
    mask = np.zeros((H, nbq, nbk), dtype=bool)
    for h in range(H):
        for I in range(nbq):
            sel = select_row(probs[h, I], tau, rho)
            mask[h, I, sel.order[: sel.n_keep]] = True
    if force_q is not None:
        mask[:, np.asarray(force_q).astype(bool), :] = True
    if force_k is not None:
        mask[:, :, np.asarray(force_k).astype(bool)] = True
    return mask


def predict_mask(q, k, b: int, tau: float, rho: float, score_scale: Optional[float] = None,
                 force_q=None, force_k=None, b_k: Optional[int] = None) -> np.ndarray:
    """Steps 1-4 chained: Q, K [H, N, d] -> block mask.  b_k, if given, is a separate block size
    for the keys (the appendix's learned-projection ablation pools queries by 128 and keys by 64);
    the mask is then [H, ceil(N/b), ceil(N/b_k)]."""
    d = np.asarray(q).shape[-1]
    if score_scale is None:
        score_scale = 1.0 / math.sqrt(d)
    probs = block_softmax(block_logits(pool_blocks(q, b), pool_blocks(k, b if b_k is None else b_k), score_scale))
    return select_blocks(probs, tau, rho, force_q, force_k)


def mask_to_index_lists(mask: np.ndarray):
    """Ascending kept key-block indices per row and their counts:
    kv_idx [H, NBq, NBk] (entries past the count are -1), kv_cnt [H, NBq]."""
    H, nbq, nbk = mask.shape
    kv_idx = np.full((H, nbq, nbk), -1, dtype=np.int32)
    kv_cnt = mask.sum(axis=-1).astype(np.int32)
    for h in range(H):
        for I in range(nbq):
            js = np.flatnonzero(mask[h, I])
            kv_idx[h, I, : js.size] = js
    return kv_idx, kv_cnt


def mask_to_bits(mask: np.ndarray) -> np.ndarray:
    """Pack mask rows into uint32 words, bit (J % 32) of word J // 32."""
    H, nbq, nbk = mask.shape
    words = (nbk + 31) // 32
    bits = np.zeros((H, nbq, words), dtype=np.uint32)
    for J in range(nbk):
        bits[:, :, J // 32] |= mask[:, :, J].astype(np.uint32) << np.uint32(J % 32)
    return bits


# --------------------------------------------------------------------------- step 5
def sparse_attention(
    q: np.ndarray,
    k: np.ndarray,
    v: np.ndarray,
    mask: np.ndarray,
    b: int,
    softmax_scale: Optional[float] = None,
    q_blocks: Optional[Iterable[int]] = None,
    heads: Optional[Sequence[int]] = None,
    return_lse: bool = False,
    b_k: Optional[int] = None,
    n_first: Optional[int] = None,
):
    """Eq. (2) with excluded (not zeroed) masked entries.

    b is the query block size; key blocks have size b_k (default b), so mask is
    [H, ceil(N/b), ceil(N/b_k)].  With n_first the blocks are those of block_ranges(N, ., n_first)
    (Sec. 4.2: two separately blocked parts) and mask has one row / column per such block.

    For token i of query block I the softmax runs over exactly the keys j < N
    that lie in key blocks J with mask[h, I, J] set; o_i is the resulting
    convex combination of those v_j.  Logits are q_i . k_j / sqrt(d_h) unless
    a scale is given.  q_blocks / heads restrict which outputs are computed
    (others stay NaN), so large shapes can be checked on a sample.
    Returns O [H, N, d] (and the natural-log sum-exp of each row's kept logits
    when return_lse is set).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    H, N, d = q.shape
    scale = 1.0 / math.sqrt(d) if softmax_scale is None else softmax_scale
    bk = b if b_k is None else b_k
    q_ranges = block_ranges(N, b, n_first)
    k_ranges = block_ranges(N, bk, n_first)
    nbq = len(q_ranges)
    assert mask.shape == (H, nbq, len(k_ranges))
    out = np.full((H, N, d), np.nan, dtype=np.float64)
    lse = np.full((H, N), np.nan, dtype=np.float64)
    head_list = range(H) if heads is None else heads
    block_list = list(range(nbq)) if q_blocks is None else list(q_blocks)
    for h in head_list:
        for I in block_list:
            rows = slice(*q_ranges[I])
            kept = np.flatnonzero(mask[h, I])
            cols = np.concatenate([np.arange(*k_ranges[J]) for J in kept])
            logits = scale * (q[h, rows] @ k[h, cols].T)
            m = logits.max(axis=1, keepdims=True)
            e = np.exp(logits - m)
            s = e.sum(axis=1, keepdims=True)
            out[h, rows] = (e / s) @ v[h, cols]
            lse[h, rows] = (m + np.log(s))[:, 0]
    return (out, lse) if return_lse else out


# --------------------------------------------------------------------------- step 6
def dense_attention(q, k, v, softmax_scale: Optional[float] = None, row_chunk: int = 1024,
                    return_lse: bool = False):
    """Eq. (1): softmax(Q K^T / sqrt(d_h)) V per head, every key visible.

    Rows are independent, so they are evaluated row_chunk at a time only to
    bound memory; no other blocking is applied.
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    H, N, d = q.shape
    scale = 1.0 / math.sqrt(d) if softmax_scale is None else softmax_scale
    out = np.empty((H, N, d), dtype=np.float64)
    lse = np.empty((H, N), dtype=np.float64)
    for h in range(H):
        kt = k[h].T
        for lo in range(0, N, row_chunk):
            hi = min(lo + row_chunk, N)
            logits = scale * (q[h, lo:hi] @ kt)
            m = logits.max(axis=1, keepdims=True)
            e = np.exp(logits - m)
            s = e.sum(axis=1, keepdims=True)
            out[h, lo:hi] = (e / s) @ v[h]
            lse[h, lo:hi] = (m + np.log(s))[:, 0]
    return (out, lse) if return_lse else out


# --------------------------------------------------------------------------- whole layer
def sparse_global_attention(q, k, v, b: int, tau: float, rho: float,
                            score_scale: Optional[float] = None,
                            softmax_scale: Optional[float] = None):
    """Steps 1-5 chained; returns (O, mask)."""
    mask = predict_mask(q, k, b, tau, rho, score_scale)
    return sparse_attention(q, k, v, mask, b, softmax_scale), mask


# --------------------------------------------------------------------------- special tokens (Sec. 4.2)
def select_blocks_unranked_columns(logits: np.ndarray, tau: float, rho: float,
                                   dense_k: np.ndarray, dense_q: Optional[np.ndarray] = None) -> np.ndarray:
    """Block selection when some key blocks take no part in the ranking (Sec. 4.2: the block map
    is predicted on patch tokens only; everything that touches a special token stays dense).

    Key blocks with dense_k set are removed before the block softmax, so they carry no mass and do
    not count towards B in k = floor(B (1 - rho)); the rule of Sec. 4.1 runs on the remaining
    columns; afterwards the removed columns are kept in every row, and query blocks with dense_q
    set keep every column."""
    dense_k = np.asarray(dense_k).astype(bool)
    H, nbq, nbk = logits.shape
    mask = np.ones((H, nbq, nbk), dtype=bool)
    ranked = np.flatnonzero(~dense_k)
    if ranked.size:
        sub = select_blocks(block_softmax(logits[:, :, ranked]), tau, rho)
        mask[:, :, ranked] = sub
    if dense_q is not None:
        mask[:, np.asarray(dense_q).astype(bool), :] = True
    return mask


def special_token_attention(q, k, v, patch_idx, special_idx, b: int, tau: float, rho: float,
                            score_scale: Optional[float] = None, softmax_scale: Optional[float] = None,
                            patch_blocks: Optional[Iterable[int]] = None, heads: Optional[Sequence[int]] = None,
                            special_rows: bool = True):
    """Sec. 4.2 as stated: split the tokens into patch tokens X_p (patch_idx, in this order) and
    special tokens X_s (special_idx).  The block map is predicted from X_p alone (pooling, block
    scores, selection over blocks of b consecutive entries of patch_idx).  A patch query attends,
    in ONE softmax, to the patch keys of its kept blocks and to every special key; a special query
    attends to every token.  Returns (O [H, N, d] in the original token order, patch block mask).

    patch_blocks / heads restrict which patch query blocks are evaluated (others stay NaN);
    special_rows = False skips the special queries."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    patch_idx = np.asarray(patch_idx, dtype=np.int64)
    special_idx = np.asarray(special_idx, dtype=np.int64)
    H, N, d = q.shape
    assert patch_idx.size + special_idx.size == N
    assert np.array_equal(np.sort(np.concatenate([patch_idx, special_idx])), np.arange(N))
    scale = 1.0 / math.sqrt(d) if softmax_scale is None else softmax_scale
    head_list = list(range(H)) if heads is None else list(heads)
    qp, kp = q[:, patch_idx], k[:, patch_idx]
    mask = predict_mask(qp, kp, b, tau, rho, score_scale)
    n_p = patch_idx.size
    nbp = num_blocks(n_p, b)
    out = np.full((H, N, d), np.nan, dtype=np.float64)
    block_list = list(range(nbp)) if patch_blocks is None else list(patch_blocks)
    for h in head_list:
        for I in block_list:
            rows = patch_idx[I * b: min((I + 1) * b, n_p)]
            kept = np.flatnonzero(mask[h, I])
            cols = np.concatenate([patch_idx[J * b: min((J + 1) * b, n_p)] for J in kept] + [special_idx])
            logits = scale * (q[h, rows] @ k[h, cols].T)
            e = np.exp(logits - logits.max(axis=1, keepdims=True))
            out[h, rows] = (e / e.sum(axis=1, keepdims=True)) @ v[h, cols]
        if special_rows and special_idx.size:
            logits = scale * (q[h, special_idx] @ k[h].T)
            e = np.exp(logits - logits.max(axis=1, keepdims=True))
            out[h, special_idx] = (e / e.sum(axis=1, keepdims=True)) @ v[h]
    return out, mask
