"""Oracle for token selection: importance scores -> top-k candidates ->
sliding-window grouping (Sections 4.2 and 4.3 of the paper).

Test infrastructure: never imported by the product path.

Readings taken where the paper is silent (all listed in the design notes):
  * the query-dimension mean is taken as a plain sum (same order of columns);
    it is added in fp32, ascending query row, one accumulator per column,
    because the sums decide an integer result (which tokens are candidates)
    and the device kernel must be able to reproduce every bit of them;
  * k = floor(T * ratio), ratio given in basis points, T = chunk tokens only;
  * ties in the top-k go to the lower token index;
  * a window that runs past the last chunk token is cut off at T and is held
    to the same threshold; windows ignore chunk boundaries;
  * tau = ceil(5 w / 8) when not given (5 at the paper's default w = 8);
  * grouping neither trims nor pads the result to the ratio;
  * the user-query slots are always appended (they have no precomputed KV);
  * scores taken from the batched per-chunk attention tensors: heads are averaged
    first (Section 3 works with head-averaged maps; Section 4.2 does not say), as
    the ascending fp32 sum over heads times the fp32 value of 1/H, then the
    query rows are summed as above.  How the head mean is rounded is not fixed
    by the paper: parity unpinned beyond the pins of block_scores below.
"""
from __future__ import annotations

import numpy as np


def default_tau(window: int) -> int:
    """Density threshold for a window of ``window`` tokens: the paper's 5-of-8,
    scaled and rounded up."""
    return (5 * window + 7) // 8


def column_scores(attn: np.ndarray) -> np.ndarray:
    """Importance score per chunk token (Section 4.2): the query->chunk block
    [Q_a, T] reduced over its query rows.  fp32, rows added in ascending order."""
    attn = np.asarray(attn, dtype=np.float32)
    s = np.zeros(attn.shape[1], dtype=np.float32)
    for q in range(attn.shape[0]):
        s = s + attn[q]          # elementwise fp32 add: one accumulator per column
    return s


def block_scores(blocks) -> np.ndarray:
    """Importance scores from the auxiliary model's batched last-layer attention
    (Section 4.2): ``blocks`` is a sequence of (A, col0, length) with A of shape
    [heads, query rows, key columns] for `chunk c + query`; the query->chunk
    block is columns col0 .. col0+length-1 (prefix columns before it and the
    query's own columns behind it are left out).  Per chunk token: mean over
    heads, then sum over query rows; the chunks' scores are concatenated."""
    out = []
    for A, col0, length in blocks:
        A = np.asarray(A, dtype=np.float32)
        H, Q_a = A.shape[0], A.shape[1]
        inv_h = np.float32(1.0) / np.float32(H)
        s = np.zeros(length, dtype=np.float32)
        for q in range(Q_a):
            m = np.zeros(length, dtype=np.float32)
            for h in range(H):
                m = m + A[h, q, col0:col0 + length]     # fp32, ascending head
            s = s + m * inv_h                           # fp32, ascending query row
        out.append(s)
    return np.concatenate(out)


def select_from_scores(s: np.ndarray, recomp_bp: int, window: int, tau: int = 0,
                       grouping: bool = True, idx_offset: int = 0, n_tail: int = 0) -> np.ndarray:
    """Top-k, grouping and output of ``select`` for a given score vector."""
    T = s.shape[0]
    cand = top_k_candidates(s, candidate_count(T, recomp_bp))
    chosen = group_windows(cand, window, tau if tau > 0 else default_tau(window)) if grouping else cand
    rel = np.nonzero(chosen)[0]
    tail = idx_offset + T + np.arange(n_tail)
    return np.concatenate([rel + idx_offset, tail]).astype(np.int32)


def candidate_count(T: int, recomp_bp: int) -> int:
    return (T * int(recomp_bp)) // 10000


def top_k_candidates(scores: np.ndarray, k: int) -> np.ndarray:
    """Boolean mask [T] of the k highest-scoring tokens (Section 4.2); equal
    scores are ranked by ascending index."""
    T = scores.shape[0]
    order = sorted(range(T), key=lambda t: (-float(scores[t]), t))
    cand = np.zeros(T, dtype=bool)
    cand[order[:k]] = True
    return cand


def group_windows(cand: np.ndarray, window: int, tau: int) -> np.ndarray:
    """Sliding-window grouping (Section 4.3).  A window of ``window`` tokens,
    step 1, is evaluated only where its first token is a candidate; if it holds
    at least ``tau`` candidates every token in it joins the result.  Candidates
    that no such window covers are dropped."""
    T = cand.shape[0]
    final = np.zeros(T, dtype=bool)
    for st in range(T):
        if not cand[st]:
            continue
        en = min(st + window, T)
        if int(cand[st:en].sum()) >= tau:
            final[st:en] = True
    return final


def select(attn: np.ndarray, recomp_bp: int, window: int, tau: int = 0,
           grouping: bool = True, idx_offset: int = 0, n_tail: int = 0) -> np.ndarray:
    """Whole selection step.  Returns the int32 cache slots to recompute,
    strictly ascending: ``idx_offset + t`` for each chosen chunk token t, then
    the ``n_tail`` slots that follow the last chunk token."""
    T = attn.shape[1]
    s = column_scores(attn)
    k = candidate_count(T, recomp_bp)
    cand = top_k_candidates(s, k)
    if grouping:
        chosen = group_windows(cand, window, tau if tau > 0 else default_tau(window))
    else:
        chosen = cand
    rel = np.nonzero(chosen)[0]
    tail = idx_offset + T + np.arange(n_tail)
    return np.concatenate([rel + idx_offset, tail]).astype(np.int32)
