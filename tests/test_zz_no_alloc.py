"""cc_select_noalloc (static device scratch, no context, no allocation) against cc_select."""
import numpy as np
import pytest
import torch

import paper_2510_10129_amd as cc
from paper_2510_10129_amd import _lib

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _both(ctx, A, bp, w, tau, flags, off, tail):
    At = torch.from_numpy(A).to(DEV)
    T = A.shape[1]
    ref_idx, ref_n = ctx.select(At, bp, w, tau, flags, off, tail)
    idx = torch.full((T + tail,), -7, dtype=torch.int32, device=DEV)
    n = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    before = torch.cuda.memory_allocated()
    cc.select_noalloc(At, bp, w, tau, flags, off, tail, idx, n)
    assert torch.cuda.memory_allocated() == before          # torch's allocator was not asked for anything
    torch.cuda.synchronize()
    got_n = int(n.item())
    assert got_n == ref_n
    assert torch.equal(idx[:got_n], ref_idx[:ref_n])
    assert bool((idx[got_n:] == -7).all())                  # nothing written past the count
    return got_n


def test_without_any_context():
    """A process that never created a context: the scratch address is resolved on first use."""
    rng = np.random.default_rng(22)
    A = rng.random((7, 3000), dtype=np.float32)
    At = torch.from_numpy(A).to(DEV)
    idx = torch.empty(3000 + 4, dtype=torch.int32, device=DEV)
    n = torch.empty(1, dtype=torch.int32, device=DEV)
    cc.select_noalloc(At, 2500, 8, 0, 0, 10, 4, idx, n)
    torch.cuda.synchronize()
    ctx = cc.Context(d=256, H_q=4, H_kv=2, d_h=64, f=1024, rope_base=1e4, rms_eps=1e-5,
                     N_cap=64, M_cap=8, T_cap=4096)
    ref_idx, ref_n = ctx.select(At, 2500, 8, 0, 0, 10, 4)
    assert int(n.item()) == ref_n and torch.equal(idx[:ref_n], ref_idx[:ref_n])
    ctx.close()


def test_two_calls_in_a_row_the_second_smaller_and_the_size_limit():
    ctx = cc.Context(d=256, H_q=4, H_kv=2, d_h=64, f=1024, rope_base=1e4, rms_eps=1e-5,
                     N_cap=1024, M_cap=64, T_cap=131072)
    rng = np.random.default_rng(21)
    big = rng.random((24, 40000), dtype=np.float32)
    big[:, 5000:5600] += 1.0                                 # a dense stretch, so that grouping keeps runs
    n1 = _both(ctx, big, 2000, 16, 0, 0, 64, 128)
    # a smaller request right after: the scratch still holds the larger one's scores above T
    small = rng.integers(0, 4, size=(5, 777)).astype(np.float32) * 0.25      # heavy ties
    n2 = _both(ctx, small, 3000, 8, 5, 0, 3, 9)
    n3 = _both(ctx, small[:, :65], 5000, 4, 2, _lib.FLAG_NO_GROUPING, 0, 0)
    assert n1 > 128 and n2 > 9 and n3 == 32
    # at the scratch capacity, and one past it
    cap = rng.random((2, 131072), dtype=np.float32)
    _both(ctx, cap, 1000, 16, 0, 0, 0, 5)
    over = torch.zeros((1, 131073), dtype=torch.float32, device=DEV)
    idx = torch.zeros(131073, dtype=torch.int32, device=DEV)
    n = torch.zeros(1, dtype=torch.int32, device=DEV)
    with pytest.raises(cc.CacheClipError) as e:
        cc.select_noalloc(over, 1000, 16, 0, 0, 0, 0, idx, n)
    assert e.value.status == _lib.CC_ERR_WORKSPACE and "131072" in str(e.value)
    with pytest.raises(cc.CacheClipError) as e:
        cc.select_noalloc(over[:, :64], 1000, 0, 0, 0, 0, 0, idx, n)
    assert e.value.status == _lib.CC_ERR_SHAPE
    ctx.close()
