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
