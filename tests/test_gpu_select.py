"""GPU parity of cc_select against the oracle: bit-exact scores, indices, count."""
import numpy as np
import pytest
import torch

import paper_2510_10129_amd as cc
from paper_2510_10129_amd import _lib
from oracle import select as osel
from workloads import CONFIGS, gen

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def ctx():
    c = cc.Context(d=256, H_q=4, H_kv=2, d_h=64, f=1024, rope_base=1e4, rms_eps=1e-5,
                   N_cap=1024, M_cap=64, T_cap=131072)
    yield c
    c.close()


def _run(ctx, A, bp, w, tau=0, flags=0, off=0, tail=0):
    At = torch.from_numpy(A).to(DEV)
    idx, n = ctx.select(At, bp, w, tau, flags, off, tail)
    return idx[:n].cpu().numpy(), n


def _check(ctx, A, bp, w, tau=0, grouping=True, off=0, tail=0):
    got, n = _run(ctx, A, bp, w, tau, 0 if grouping else _lib.FLAG_NO_GROUPING, off, tail)
    ref = osel.select(A, bp, w, tau, grouping, off, tail)
    assert n == len(ref)
    assert np.array_equal(got, ref)
    return n


def test_scores_bit_exact(ctx):
    rng = np.random.default_rng(0)
    for Qa, T in ((1, 1), (3, 65), (32, 1024), (100, 777), (128, 16384)):
        A = rng.random((Qa, T), dtype=np.float32)
        At = torch.from_numpy(A).to(DEV)
        s = torch.empty(T, dtype=torch.float32, device=DEV)
        ctx.step_column_scores(At, s)
        assert np.array_equal(s.cpu().numpy().view(np.uint32), osel.column_scores(A).view(np.uint32))


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_configs_bit_exact(ctx, name):
    wl = CONFIGS[name]
    A = gen.aux_attention(wl)
    for bp in wl.recomp_bp:
        n = _check(ctx, A, bp, wl.window, wl.tau, True, wl.P, wl.Q)
        print(f"{name} recomp {bp / 100:.0f}%: k={wl.T * bp // 10000} -> M={n} (M_sel/T={(n - wl.Q) / wl.T:.3f})")
    _check(ctx, A, wl.recomp_bp[0], wl.window, wl.tau, False, wl.P, wl.Q)


def test_random_ragged_with_heavy_ties(ctx):
    rng = np.random.default_rng(1)
    for it in range(40):
        T = int(rng.integers(1, 6000))
        Qa = int(rng.integers(1, 9))
        w = int(rng.integers(1, 70))
        tau = int(rng.integers(0, w + 1))
        bp = int(rng.choice([0, 1, 500, 2000, 5000, 9999, 10000]))
        A = rng.integers(0, 4, size=(Qa, T)).astype(np.float32) * 0.25     # few distinct sums
        _check(ctx, A, bp, w, tau, bool(it % 3), int(rng.integers(0, 100)), int(rng.integers(0, 40)))


def test_degenerate_cases(ctx):
    A = np.full((4, 300), 0.125, dtype=np.float32)           # all equal: lowest indices win
    got, n = _run(ctx, A, 2000, 8, 5, off=10, tail=3)
    # k = 60 candidates 0..59; the last passing window starts at 55 (55..59 = 5 candidates) and ends at 62
    assert got.tolist() == list(range(10, 73)) + [310, 311, 312]
    assert np.array_equal(got, osel.select(A, 2000, 8, 5, True, 10, 3))
    _check(ctx, A, 0, 8, 5, True, 0, 0)                      # nothing at all
    _check(ctx, A, 10000, 8, 5, True, 0, 0)                  # everything
    _check(ctx, np.zeros((2, 50), np.float32), 5000, 8)      # zeros incl. default tau
    neg = np.zeros((1, 64), np.float32); neg[0, ::2] = -0.0
    _check(ctx, neg, 2500, 4, 2)                             # -0 == +0
    wide = np.random.default_rng(3).random((2, 5000)).astype(np.float32)
    _check(ctx, wide, 3000, 1024, 300)                       # widest window
    _check(ctx, wide[:, :7], 5000, 32, 2)                    # window longer than T
    big = np.random.default_rng(4).random((2, 131072)).astype(np.float32)
    _check(ctx, big, 2000, 16)                               # T at capacity


def test_long_inputs_with_ties_and_crowded_threshold_digit(ctx):
    """Paths of the selection kernel that short inputs do not reach: more keys share the
    threshold's leading digit than its LDS list holds (the remaining digits then come from further
    passes over the scores), with and without equal scores at the threshold."""
    rng = np.random.default_rng(6)
    T = 100000
    few = rng.integers(1, 5, size=(3, T)).astype(np.float32) * 0.125           # ten distinct sums: crowded, tied
    _check(ctx, few, 2000, 16, 0, True, 7, 3)
    _check(ctx, few, 5000, 8, 5, False, 0, 0)
    narrow = (1.0 + rng.random((1, T)) * 0.1).astype(np.float32)                 # one binade, all distinct (mostly)
    _check(ctx, narrow, 2000, 16, 0, True, 0, 0)
    mixed = narrow.copy()
    mixed[0, ::3] = np.float32(1.05)                                            # a third of the keys equal, threshold among them
    _check(ctx, mixed, 5000, 32, 0, True, 64, 128)


def test_strided_input_and_async_count(ctx):
    rng = np.random.default_rng(5)
    full = torch.from_numpy(rng.random((16, 1000), dtype=np.float32)).to(DEV)
    view = full[:, 100:740]                                  # ld = 1000, T = 640
    idx, n = ctx.select(view, 2000, 8, 5, 0, 0, 0)
    ref = osel.select(view.cpu().numpy(), 2000, 8, 5)
    assert n == len(ref) and np.array_equal(idx[:n].cpu().numpy(), ref)
    n_out = torch.zeros(1, dtype=torch.int32, device=DEV)
    idx2, none = ctx.select(view, 2000, 8, 5, n_out=n_out, sync=False)
    torch.cuda.synchronize()
    assert none is None and int(n_out.item()) == n and torch.equal(idx2[:n], idx[:n])


def test_argument_errors(ctx):
    A = torch.zeros((2, 64), dtype=torch.float32, device=DEV)
    for kw, code in ((dict(recomp_bp=10001, window=8), _lib.CC_ERR_SHAPE),
                     (dict(recomp_bp=100, window=0), _lib.CC_ERR_SHAPE),
                     (dict(recomp_bp=100, window=2000), _lib.CC_ERR_SHAPE),
                     (dict(recomp_bp=100, window=8, tau=9), _lib.CC_ERR_SHAPE),
                     (dict(recomp_bp=100, window=8, n_tail=-1), _lib.CC_ERR_SHAPE)):
        with pytest.raises(cc.CacheClipError) as e:
            ctx.select(A, **kw)
        assert e.value.status == code
    small = cc.Context(d=256, H_q=4, H_kv=2, d_h=64, f=1024, rope_base=1e4, rms_eps=1e-5,
                       N_cap=64, M_cap=8, T_cap=32)
    with pytest.raises(cc.CacheClipError) as e:
        small.select(A, 100, 8)
    assert e.value.status == _lib.CC_ERR_WORKSPACE
    small.close()


# ------------------------------------------------- scores from batched per-chunk attention
def _dev_blocks(blocks_np, pad_rows=0, pad_cols=0):
    """Device copies; with padding the blocks become strided views of larger tensors."""
    out = []
    for A, c0, L in blocks_np:
        H, Qa, W = A.shape
        big = torch.full((H, Qa + pad_rows, W + pad_cols), 123.0, dtype=torch.float32, device=DEV)
        big[:, :Qa, :W] = torch.from_numpy(A).to(DEV)
        out.append((big[:, :Qa, :W], c0, L))
    return out


@pytest.mark.parametrize("H,Qa,P,lens", [
    (1, 1, 0, [1]),
    (3, 5, 4, [63, 64, 65, 1, 200]),
    (14, 33, 16, [300, 17, 511]),
    (16, 128, 64, [1024, 777]),
    (28, 70, 8, [129] * 5),
    (9, 64, 0, [40] * 70),            # more batch elements than one launch takes
])
def test_block_scores_bit_exact(ctx, H, Qa, P, lens):
    rng = np.random.default_rng(H * 1000 + Qa)
    blocks = [(rng.random((H, Qa, P + L + Qa), dtype=np.float32), P, L) for L in lens]
    ref = osel.block_scores(blocks)
    for pad in (0, 3):
        score = torch.full((sum(lens),), -1.0, dtype=torch.float32, device=DEV)
        ctx.step_block_scores(_dev_blocks(blocks, pad, pad), score)
        torch.cuda.synchronize()
        assert np.array_equal(score.cpu().numpy().view(np.uint32), ref.view(np.uint32)), (H, Qa, pad)


def test_select_blocks_matches_oracle(ctx):
    rng = np.random.default_rng(11)
    for H, Qa, P, lens, bp, w in ((4, 16, 8, [256] * 4, 2000, 8), (14, 32, 16, [300, 100, 511, 77], 1000, 16),
                                  (2, 3, 0, [50], 5000, 4)):
        # peaked rows: a few columns carry most of the weight, with ties across heads
        blocks = []
        for L in lens:
            A = rng.random((H, Qa, P + L + Qa), dtype=np.float32) * 0.01
            hot = rng.integers(P, P + L, size=max(1, L // 10))
            A[:, :, hot] += rng.integers(1, 4, size=(1, 1, len(hot))).astype(np.float32) * 0.25
            blocks.append((A, P, L))
        s = osel.block_scores(blocks)
        for grouping in (True, False):
            ref = osel.select_from_scores(s, bp, w, 0, grouping, P, Qa)
            idx, n = ctx.select_blocks(_dev_blocks(blocks), bp, w, 0, 0 if grouping else _lib.FLAG_NO_GROUPING, P, Qa)
            assert n == len(ref) and np.array_equal(idx[:n].cpu().numpy(), ref)


def test_block_scores_argument_errors(ctx):
    A = torch.zeros((2, 4, 40), dtype=torch.float32, device=DEV)
    score = torch.zeros(64, dtype=torch.float32, device=DEV)
    with pytest.raises(ValueError):
        ctx.step_block_scores([(A, 30, 20)], score)                     # block runs past its width
    with pytest.raises(ValueError):
        ctx.step_block_scores([(A, 0, 10), (A[:1], 0, 10)], score)      # differing head counts
    arr = (_lib._AuxBlock * 1)(_lib._AuxBlock(A.data_ptr(), A.stride(0), A.stride(1), 0, 0))
    assert ctx._lib.cc_step_block_scores(ctx._h, arr, 1, 2, 4, score.data_ptr()) == _lib.CC_ERR_SHAPE   # len 0
    arr = (_lib._AuxBlock * 1)(_lib._AuxBlock(A.data_ptr(), A.stride(0), 10, 0, 20))
    assert ctx._lib.cc_step_block_scores(ctx._h, arr, 1, 2, 4, score.data_ptr()) == _lib.CC_ERR_SHAPE   # rows overlap
    arr = (_lib._AuxBlock * 1)(_lib._AuxBlock(None, A.stride(0), A.stride(1), 0, 20))
    assert ctx._lib.cc_step_block_scores(ctx._h, arr, 1, 2, 4, score.data_ptr()) == _lib.CC_ERR_NULL
    small = cc.Context(d=256, H_q=4, H_kv=2, d_h=64, f=1024, rope_base=1e4, rms_eps=1e-5,
                       N_cap=64, M_cap=8, T_cap=32)
    with pytest.raises(cc.CacheClipError) as e:
        small.select_blocks([(A, 0, 40)], 1000, 8)
    assert e.value.status == _lib.CC_ERR_WORKSPACE
    small.close()


@pytest.mark.parametrize("name,prefix", [("C2", None), ("C2", 0), ("C4", None)])
def test_blocks_window_sweep_and_no_prefix(ctx, name, prefix):
    """Per-chunk-normalised scores from batched tensors at request size: windows 8, 16, 32,
    grouping on and off, with and without a shared prefix, ragged chunk lengths (C4)."""
    import dataclasses
    wl = CONFIGS[name]
    if name == "C4":       # a third of the request keeps the host-side generator quick
        wl = dataclasses.replace(wl, chunk_lens=wl.chunk_lens[:10], Q_a=32)
    blocks = gen.aux_attention_blocks(wl, heads=14 if name == "C2" else 9, prefix=prefix)
    P = blocks[0][1]
    s = osel.block_scores(blocks)
    assert abs(float(s.sum()) - wl.Q_a * len(blocks)) < 0.5 * wl.Q_a * len(blocks)   # most mass sits on chunk tokens
    dev_blocks = _dev_blocks(blocks)
    score = torch.empty(wl.T, dtype=torch.float32, device=DEV)
    ctx.step_block_scores(dev_blocks, score)
    assert np.array_equal(score.cpu().numpy().view(np.uint32), s.view(np.uint32))
    for w in (8, 16, 32):
        for grouping in (True, False):
            ref = osel.select_from_scores(s, 2000, w, 0, grouping, P, wl.Q)
            idx, n = ctx.select_blocks(dev_blocks, 2000, w, 0, 0 if grouping else _lib.FLAG_NO_GROUPING, P, wl.Q)
            assert n == len(ref) and np.array_equal(idx[:n].cpu().numpy(), ref), (name, prefix, w, grouping)
        print(f"{name} prefix={P} w={w}: M_sel/T = {(len(osel.select_from_scores(s, 2000, w, 0, True, P, wl.Q)) - wl.Q) / wl.T:.3f}")
