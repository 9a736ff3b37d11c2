"""Pins for the selection oracle (Sections 4.2-4.3): brute force from the set
definition, hand-worked cases, closed forms and degenerate cases."""
import itertools
import os

import numpy as np
import pytest

from oracle import select as osel
from workloads import CONFIGS, gen

GOLD = os.path.join(os.path.dirname(__file__), "golden", "grouping_examples.txt")


def _golden_cases():
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a, b, c = line.split("|")
        T, w, tau = map(int, a.split())
        yield T, w, tau, [int(v) for v in b.split()], [int(v) for v in c.split()]


@pytest.mark.parametrize("T,w,tau,cands,expect", list(_golden_cases()))
def test_grouping_hand_worked(T, w, tau, cands, expect):
    cand = np.zeros(T, dtype=bool)
    cand[cands] = True
    got = np.nonzero(osel.group_windows(cand, w, tau))[0].tolist()
    assert got == expect


def _grouping_by_membership(cand, w, tau):
    """The same rule read from the other side: token t is taken iff some start
    st in (t-w, t] is a candidate whose window [st, st+w) ∩ [0,T) holds >= tau
    candidates."""
    T = len(cand)
    cs = set(np.nonzero(cand)[0].tolist())
    out = []
    for t in range(T):
        ok = False
        for st in range(max(0, t - w + 1), t + 1):
            if st in cs and len(cs & set(range(st, min(st + w, T)))) >= tau:
                ok = True
        if ok:
            out.append(t)
    return out


def test_grouping_exhaustive_small():
    # every candidate set on 10 tokens, two window shapes
    T = 10
    for w, tau in ((3, 2), (4, 3)):
        for bits in itertools.product((False, True), repeat=T):
            cand = np.array(bits)
            got = np.nonzero(osel.group_windows(cand, w, tau))[0].tolist()
            assert got == _grouping_by_membership(cand, w, tau)


def test_grouping_random_vs_membership():
    rng = np.random.default_rng(0)
    for _ in range(50):
        T = int(rng.integers(1, 200))
        w = int(rng.integers(1, 20))
        tau = int(rng.integers(1, w + 1))
        cand = rng.random(T) < rng.random()
        got = np.nonzero(osel.group_windows(cand, w, tau))[0].tolist()
        assert got == _grouping_by_membership(cand, w, tau)


def test_grouping_invariants():
    rng = np.random.default_rng(1)
    T, w, tau = 500, 8, 5
    cand = rng.random(T) < 0.3
    fin = osel.group_windows(cand, w, tau)
    # all candidates -> everything (T >= w); fewer than tau candidates -> nothing
    assert osel.group_windows(np.ones(T, bool), w, tau).all()
    few = np.zeros(T, bool); few[[3, 100, 200, 499]] = True
    assert not osel.group_windows(few, w, tau).any()
    # every taken token lies in a passing window that starts at a candidate
    for t in np.nonzero(fin)[0]:
        assert any(cand[st] and cand[st:min(st + w, T)].sum() >= tau
                   for st in range(max(0, t - w + 1), t + 1))
    # tau = 1 keeps every candidate; runs are at least... every candidate start gives a full window
    keep = osel.group_windows(cand, w, 1)
    assert (keep | ~cand).all()


def test_default_tau():
    assert osel.default_tau(8) == 5          # the paper's default pair
    assert osel.default_tau(16) == 10 and osel.default_tau(32) == 20
    assert osel.default_tau(1) == 1 and osel.default_tau(3) == 2


def test_column_scores_closed_forms():
    A = np.ones((37, 11), dtype=np.float32)
    assert (osel.column_scores(A) == 37).all()
    # column t of row q holds q*t: sum = t * Q(Q-1)/2, exact in fp32 here
    Q, T = 16, 9
    A = (np.arange(Q)[:, None] * np.arange(T)[None, :]).astype(np.float32)
    assert (osel.column_scores(A) == np.arange(T) * (Q * (Q - 1) // 2)).all()
    # transposed operand would fail: a non-square block sums over rows, giving T values
    assert osel.column_scores(np.zeros((3, 5), np.float32)).shape == (5,)


def test_column_scores_fp32_sequential_order():
    # 1 + 2^-24 + 2^-24: added in row order in fp32 each tiny term is lost
    # (ties to even); any pairwise or fp64 summation would give 1 + 2^-23.
    A = np.array([[1.0], [2.0 ** -24], [2.0 ** -24]], dtype=np.float32)
    assert osel.column_scores(A)[0] == np.float32(1.0)
    # reversed rows: the two tiny terms add first and survive
    assert osel.column_scores(A[::-1])[0] == np.float32(1.0 + 2.0 ** -23)
    # independent replay with explicit scalar fp32 accumulation
    rng = np.random.default_rng(2)
    B = rng.random((50, 7)).astype(np.float32)
    ref = []
    for t in range(7):
        acc = np.float32(0)
        for q in range(50):
            acc = np.float32(acc + B[q, t])
        ref.append(acc)
    assert (osel.column_scores(B) == np.array(ref, dtype=np.float32)).all()


def test_topk_brute_force_and_ties():
    rng = np.random.default_rng(3)
    for _ in range(30):
        T = int(rng.integers(1, 60))
        s = rng.integers(0, 6, size=T).astype(np.float32)       # heavy ties
        k = int(rng.integers(0, T + 1))
        cand = osel.top_k_candidates(s, k)
        assert cand.sum() == k
        # definition check: nobody outside beats or ties-with-lower-index anybody inside
        ins, outs = np.nonzero(cand)[0], np.nonzero(~cand)[0]
        for i in ins:
            for o in outs:
                assert s[i] > s[o] or (s[i] == s[o] and i < o)
    s = np.full(20, 0.25, dtype=np.float32)
    assert np.nonzero(osel.top_k_candidates(s, 7))[0].tolist() == list(range(7))
    assert not osel.top_k_candidates(s, 0).any()
    assert osel.top_k_candidates(s, 20).all()
    # +0 and -0 are the same score
    s = np.array([0.0, -0.0, 0.0, 1.0], dtype=np.float32)
    assert np.nonzero(osel.top_k_candidates(s, 3))[0].tolist() == [0, 1, 3]


def test_candidate_count_floor():
    assert osel.candidate_count(1024, 2000) == 204       # Tiny config: floor(204.8)
    assert osel.candidate_count(16384, 2000) == 3276
    assert osel.candidate_count(10, 0) == 0 and osel.candidate_count(10, 10000) == 10


def test_select_end_to_end_small():
    # scores built so the candidates are known: columns 2,3,4,6,7,15 dominate
    T = 20
    A = np.full((3, T), 0.01, dtype=np.float32)
    for c in (2, 3, 4, 6, 7, 15):
        A[:, c] = 0.5
    idx = osel.select(A, recomp_bp=3000, window=8, tau=5, idx_offset=4, n_tail=2)
    assert idx.dtype == np.int32
    assert idx.tolist() == [4 + t for t in range(2, 10)] + [24, 25]
    # grouping off (the paper's ablation): candidates as they are
    idx = osel.select(A, 3000, 8, 5, grouping=False, idx_offset=4, n_tail=0)
    assert idx.tolist() == [6, 7, 8, 10, 11, 19]
    # ratio 0 -> only the query tail; ratio 100 % -> every chunk token
    assert osel.select(A, 0, 8, 5, idx_offset=4, n_tail=2).tolist() == [24, 25]
    assert osel.select(A, 10000, 8, 5, idx_offset=4, n_tail=0).tolist() == list(range(4, 24))


def test_select_on_tiny_config_properties():
    wl = CONFIGS["C1"]
    A = gen.aux_attention(wl)
    assert A.shape == (wl.Q_a, wl.T) and np.allclose(A.sum(axis=1), 1.0, atol=1e-5)
    idx = osel.select(A, 2000, wl.window, wl.tau, idx_offset=wl.P, n_tail=wl.Q)
    assert (np.diff(idx) > 0).all() and idx[0] >= wl.P and idx[-1] == wl.N - 1
    assert idx[-wl.Q:].tolist() == list(range(wl.P + wl.T, wl.N))
    # same result from an independent vectorised formulation
    s = osel.column_scores(A)
    k = 204
    order = np.lexsort((np.arange(wl.T), -s.astype(np.float64)))
    cand = np.zeros(wl.T, bool); cand[order[:k]] = True
    c = np.concatenate([[0], np.cumsum(cand)])
    ends = np.minimum(np.arange(wl.T) + wl.window, wl.T)
    passing = cand & ((c[ends] - c[np.arange(wl.T)]) >= wl.tau)
    marked = np.zeros(wl.T, bool)
    for st in np.nonzero(passing)[0]:
        marked[st:st + wl.window] = True
    assert idx[:-wl.Q].tolist() == (np.nonzero(marked)[0] + wl.P).tolist()


# ------------------------------------------------- scores from batched per-chunk attention
def _raw_blocks(rng, H, Q_a, lens, P, pad=0):
    blocks = []
    for L in lens:
        W = P + L + Q_a + pad
        A = rng.random((H, Q_a, W), dtype=np.float32)
        blocks.append((A, P, L))
    return blocks


def test_block_scores_closed_forms_and_exclusions():
    rng = np.random.default_rng(0)
    # all ones, power-of-two head count: head mean is exactly 1, the score exactly Q_a
    ones = [(np.ones((8, 5, 40), np.float32), 7, 20), (np.ones((8, 5, 33), np.float32), 7, 11)]
    s = osel.block_scores(ones)
    assert s.shape == (31,) and np.all(s == 5.0)
    # a single head: the head mean is the block itself, so the scores are the column sums
    b1 = _raw_blocks(rng, 1, 9, [17, 64, 3], 4)
    ref = np.concatenate([osel.column_scores(A[0][:, c0:c0 + L]) for A, c0, L in b1])
    assert np.array_equal(osel.block_scores(b1), ref)
    # what lies outside the query->chunk block (prefix and query columns) does not matter
    b2 = _raw_blocks(rng, 3, 6, [10, 25], 5)
    base = osel.block_scores(b2)
    for A, c0, L in b2:
        A[:, :, :c0] = 99.0
        A[:, :, c0 + L:] = -7.0
    assert np.array_equal(osel.block_scores(b2), base)
    # chunks are concatenated in order
    assert np.array_equal(osel.block_scores(b2[::-1]), np.concatenate([base[10:], base[:10]]))


def test_block_scores_match_float64_mean_then_sum():
    rng = np.random.default_rng(1)
    for H, Q_a in ((3, 7), (14, 33), (16, 128), (28, 5)):
        blocks = _raw_blocks(rng, H, Q_a, [50, 129], 6)
        got = osel.block_scores(blocks).astype(np.float64)
        ref = np.concatenate([A[:, :, c0:c0 + L].astype(np.float64).mean(axis=0).sum(axis=0) for A, c0, L in blocks])
        # fp32 accumulation of H + Q_a terms of size <= 1 and Q_a respectively
        assert np.max(np.abs(got - ref)) <= 1e-6 * Q_a * (1 + H / 8)
    # a head that carries weight w in one (q, column) entry adds w / H to that column only
    A = np.zeros((4, 3, 20), np.float32)
    A[2, 1, 9] = 0.5
    s = osel.block_scores([(A, 2, 15)])
    assert s[7] == np.float32(0.125) and np.count_nonzero(s) == 1


def test_select_from_scores_equals_select():
    rng = np.random.default_rng(2)
    A = rng.random((6, 300), dtype=np.float32)
    for bp, w, tau, grp in ((2000, 8, 5, True), (500, 16, 0, True), (3000, 8, 5, False)):
        assert np.array_equal(osel.select_from_scores(osel.column_scores(A), bp, w, tau, grp, 11, 4),
                              osel.select(A, bp, w, tau, grp, 11, 4))
