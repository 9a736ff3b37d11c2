"""GPU parity of cc_assemble_cache (Section 4.1: concatenation behind one prefix copy,
keys re-numbered to global positions) against the oracle's concat_caches.

Copies (prefix rows, every value row, chunk 0's keys, the zeroed tail) are bit-exact.
Re-rotated keys are floating point: the device turns bf16 keys in fp32 and rounds to
bf16, the oracle in fp64; the bound is half a bf16 spacing of the exact result plus
fp32 rounding noise, written below as 2^-8 of the row's largest magnitude."""
import numpy as np
import pytest
import torch

import paper_2510_10129_amd as cc
from paper_2510_10129_amd import _lib
from oracle import bf16 as obf
from oracle import fixture, layer
from workloads import CONFIGS, ModelShape, gen

from _gpu_util import DEV, bits_f64, dev_bf16, host_bits

pytestmark = pytest.mark.gpu


def _ctx(model, N):
    return cc.Context.for_model(model, N_cap=N, M_cap=1, T_cap=64)


def _assemble(model, chunk_K_bits, chunk_V_bits, P, Q, pad_rows=0):
    T = sum(k.shape[0] - P for k in chunk_K_bits)
    N = P + T + Q + pad_rows
    ctx = _ctx(model, N)
    Kd = torch.full((N, model.H_kv, model.d_h), 7.0, dtype=torch.bfloat16, device=DEV)
    Vd = torch.full((N, model.H_kv, model.d_h), 7.0, dtype=torch.bfloat16, device=DEV)
    ctx.assemble_cache([dev_bf16(k) for k in chunk_K_bits], [dev_bf16(v) for v in chunk_V_bits], P, Q,
                       cc.KVLayer(Kd, Vd))
    torch.cuda.synchronize()
    ctx.close()
    return host_bits(Kd), host_bits(Vd)


def _check(model, chunk_K_bits, chunk_V_bits, P, Q, Kg, Vg, pad_rows=0):
    """Against the definition: prefix once, chunks appended, keys turned by start_c."""
    pos = 0
    assert np.array_equal(Kg[:P], chunk_K_bits[0][:P]) and np.array_equal(Vg[:P], chunk_V_bits[0][:P])
    start = 0
    for c, (Kc, Vc) in enumerate(zip(chunk_K_bits, chunk_V_bits)):
        L = Kc.shape[0] - P
        rows = slice(P + start, P + start + L)
        assert np.array_equal(Vg[rows], Vc[P:]), c
        if start == 0:
            assert np.array_equal(Kg[rows], Kc[P:])
        else:
            ref = layer.rope_rotate(obf.bits_to_f64(Kc[P:]), np.full(L, start), model.rope_base)
            err = np.abs(bits_f64(Kg[rows]) - ref)
            assert err.max() <= 2.0 ** -8 * np.abs(ref).max(), (c, err.max())
            # and the bf16 codes are the oracle's except where the exact value sits next to a tie
            same = (Kg[rows] == obf.f64_to_bits(ref)).mean()
            assert same > 0.995, (c, same)
        start += L
    T = start
    assert not Kg[P + T:P + T + Q].any() and not Vg[P + T:P + T + Q].any()
    if pad_rows:          # rows past the tail are not touched
        assert (Kg[P + T + Q:] == 0x40E0).all() and (Vg[P + T + Q:] == 0x40E0).all()


def test_real_chunk_caches_against_concat_caches():
    model = ModelShape(128, 4, 2, 64, 192, 1e4, 1e-5, False, 1)
    ws = [gen.layer_weights(model, 0, seed=41)]
    P, lens, Q = 5, (33, 7, 64, 18), 6
    n = P + sum(lens) + Q
    xb = gen.f32_to_bf16_bits(np.random.default_rng(42).standard_normal((n, model.d)).astype(np.float32))
    per = fixture.chunk_caches(xb, P, lens, ws, model)
    Kref, Vref = fixture.concat_caches(per, P, lens, Q, model, 1)
    cK, cV = [p[0][0] for p in per], [p[1][0] for p in per]
    Kg, Vg = _assemble(model, cK, cV, P, Q, pad_rows=3)
    _check(model, cK, cV, P, Q, Kg, Vg, pad_rows=3)
    assert np.array_equal(Vg[:n], Vref[0])
    assert (Kg[:n] == Kref[0]).mean() > 0.995


@pytest.mark.parametrize("H_kv,d_h,P,Q,n_chunks", [(8, 128, 64, 128, 16), (1, 64, 0, 0, 3), (4, 128, 16, 5, 70)])
def test_random_store_shapes(H_kv, d_h, P, Q, n_chunks):
    """Llama-3-8B cache rows at the 16k layout; no prefix and no tail; more chunks than one launch takes."""
    rng = np.random.default_rng(n_chunks)
    model = ModelShape(H_kv * d_h, H_kv, H_kv, d_h, 64, 5e5, 1e-5, False, 1)
    lens = [1024] * n_chunks if n_chunks == 16 else [int(v) for v in rng.integers(1, 90, size=n_chunks)]
    cK = [gen.f32_to_bf16_bits(rng.standard_normal((P + L, H_kv, d_h)).astype(np.float32)) for L in lens]
    cV = [gen.f32_to_bf16_bits(rng.standard_normal((P + L, H_kv, d_h)).astype(np.float32)) for L in lens]
    Kg, Vg = _assemble(model, cK, cV, P, Q)
    _check(model, cK, cV, P, Q, Kg, Vg)


def test_argument_errors():
    model = ModelShape(128, 2, 2, 64, 64, 1e4, 1e-5, False, 1)
    ctx = _ctx(model, 40)
    K = torch.zeros((20, 2, 64), dtype=torch.bfloat16, device=DEV)
    dst = cc.KVLayer(torch.zeros((40, 2, 64), dtype=torch.bfloat16, device=DEV),
                     torch.zeros((40, 2, 64), dtype=torch.bfloat16, device=DEV))
    with pytest.raises(cc.CacheClipError) as e:
        ctx.assemble_cache([K, K, K], [K, K, K], 4, 0, dst)          # 4 + 3*16 > 40
    assert e.value.status == _lib.CC_ERR_SHAPE
    with pytest.raises(cc.CacheClipError) as e:
        ctx.assemble_cache([K[:4]], [K[:4]], 4, 0, dst)              # chunk of length 0
    assert e.value.status == _lib.CC_ERR_SHAPE
    ctx.assemble_cache([K, K], [K, K], 4, 4, dst)                    # fits exactly: 4 + 32 + 4
    torch.cuda.synchronize()
    ctx.close()
