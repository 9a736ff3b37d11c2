"""Pins for the layer oracle: closed forms, library routines (torch CPU SDPA,
rms_norm, silu), the paper's two end points (recompute everything == full
attention prefill, recompute nothing == plain concatenation) and invariants."""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import bf16, fixture, layer
from workloads import CONFIGS, ModelShape, gen

SMALL = ModelShape(d=64, H_q=4, H_kv=2, d_h=16, f=128, rope_base=100.0, rms_eps=1e-5,
                   qkv_bias=True, n_layers=1)


def _weights(model, seed=0, layer_id=0):
    return gen.layer_weights(model, layer_id, seed)


def _x_bits(n, d, seed):
    r = np.random.default_rng(seed)
    return gen.f32_to_bf16_bits(r.standard_normal((n, d)).astype(np.float32))


# ---------------------------------------------------------------- bf16
def test_bf16_rounding_hand_cases():
    r = bf16.round_f64
    assert r(np.array([1 + 2.0 ** -8]))[0] == 1.0                       # tie -> even (down)
    assert r(np.array([1 + 3 * 2.0 ** -8]))[0] == 1 + 2.0 ** -6         # tie -> even (up)
    assert r(np.array([1 + 2.0 ** -8 + 2.0 ** -30]))[0] == 1 + 2.0 ** -7
    # no double rounding through fp32: fp32 would first drop the 2^-40 and then tie down
    assert r(np.array([1 + 2.0 ** -8 + 2.0 ** -40]))[0] == 1 + 2.0 ** -7
    assert r(np.array([-3.0, 0.0, 0.5]))[...].tolist() == [-3.0, 0.0, 0.5]
    assert bf16.f64_to_bits(np.array([1.0, -2.0, 0.0])).tolist() == [0x3F80, 0xC000, 0x0000]
    assert bf16.bits_to_f64(np.array([0x3F80, 0x4049], np.uint16)).tolist() == [1.0, 3.140625]


def test_bf16_matches_torch_on_fp32_inputs():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 3
    ours = bf16.f64_to_bits(x.astype(np.float64))
    theirs = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert (ours == theirs).all()
    assert (ours == gen.f32_to_bf16_bits(x)).all()
    assert (bf16.bits_to_f64(ours) == gen.bf16_to_f32(ours).astype(np.float64)).all()


# ---------------------------------------------------------------- pieces
def test_rope_closed_forms():
    # d_h = 4, base = 4: inverse frequencies 1 and 4**-0.5 = 0.5; pairs (0,2) and (1,3)
    e0 = np.array([[[1.0, 0, 0, 0]]])
    e1 = np.array([[[0, 1.0, 0, 0]]])
    out0 = layer.rope_rotate(e0, np.array([1]), 4.0)[0, 0]
    out1 = layer.rope_rotate(e1, np.array([1]), 4.0)[0, 0]
    assert np.allclose(out0, [math.cos(1), 0, math.sin(1), 0], atol=1e-15)
    assert np.allclose(out1, [0, math.cos(0.5), 0, math.sin(0.5)], atol=1e-15)
    # a vector on the second half turns towards minus the first half
    e2 = np.array([[[0, 0, 1.0, 0]]])
    assert np.allclose(layer.rope_rotate(e2, np.array([1]), 4.0)[0, 0],
                       [-math.sin(1), 0, math.cos(1), 0], atol=1e-15)
    # position 0 is the identity
    x = np.random.default_rng(0).standard_normal((3, 2, 8))
    assert np.array_equal(layer.rope_rotate(x, np.zeros(3), 50.0), x)


def test_rope_vs_complex_exponential_and_invariants():
    rng = np.random.default_rng(1)
    d_h, base = 16, 1.0e4
    x = rng.standard_normal((5, 3, d_h))
    pos = np.array([0, 1, 7, 100, 4095])
    got = layer.rope_rotate(x, pos, base)
    half = d_h // 2
    z = x[..., :half] + 1j * x[..., half:]
    theta = np.array([base ** (-2 * j / d_h) for j in range(half)])
    zr = z * np.exp(1j * pos[:, None, None] * theta[None, None, :])
    assert np.allclose(got[..., :half], zr.real, atol=1e-12)
    assert np.allclose(got[..., half:], zr.imag, atol=1e-12)
    # norms are kept; rotations add; q.k depends only on the position difference
    assert np.allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(x, axis=-1))
    twice = layer.rope_rotate(layer.rope_rotate(x, pos, base), np.full(5, 9), base)
    assert np.allclose(twice, layer.rope_rotate(x, pos + 9, base), atol=1e-10)
    q, k = rng.standard_normal((1, 1, d_h)), rng.standard_normal((1, 1, d_h))
    def dot(pq, pk):
        return float((layer.rope_rotate(q, np.array([pq]), base) *
                      layer.rope_rotate(k, np.array([pk]), base)).sum())
    assert abs(dot(10, 3) - dot(1010, 1003)) < 1e-9
    assert abs(dot(10, 3) - dot(3, 10)) > 1e-3


def test_rmsnorm_and_silu_closed_forms():
    w = np.array([1.0, 2.0, 3.0, 4.0])
    x = np.full((1, 4), 5.0)
    # constant row, eps = 0: x/rms = 1 -> output = w
    assert np.allclose(layer.rmsnorm(x, w, 0.0), w)
    x = np.array([[3.0, 4.0, 0.0, 0.0]])            # mean square = 25/4
    assert np.allclose(layer.rmsnorm(x, np.ones(4), 0.0), x / 2.5)
    assert np.allclose(layer.rmsnorm(x, np.ones(4), 0.75), x / math.sqrt(7.0))
    xt = torch.randn(6, 32, dtype=torch.float64)
    wt = torch.randn(32, dtype=torch.float64)
    assert np.allclose(layer.rmsnorm(xt.numpy(), wt.numpy(), 1e-5),
                       F.rms_norm(xt, (32,), wt, 1e-5).numpy(), atol=1e-12)
    assert layer.silu(np.array([0.0]))[0] == 0.0
    assert abs(layer.silu(np.array([1.0]))[0] - 1 / (1 + math.exp(-1))) < 1e-15
    assert np.allclose(layer.silu(xt.numpy()), F.silu(xt).numpy(), atol=1e-12)


# ---------------------------------------------------------------- whole layer vs torch
def _torch_layer(x_bits, pos, w, model):
    """Same decoder layer from torch CPU library routines, fp64; rotary done as
    a complex multiplication; K/V rounded to bf16 through torch's converter."""
    t = lambda name: torch.from_numpy(bf16.bits_to_f64(w[name]))
    x = torch.from_numpy(bf16.bits_to_f64(x_bits))
    n = x.shape[0]
    h = F.rms_norm(x, (model.d,), t("w_in_norm"), model.rms_eps)
    qkv = F.linear(h, t("w_qkv"), t("b_qkv") if w["b_qkv"] is not None else None)
    nq, nk = model.H_q * model.d_h, model.H_kv * model.d_h
    q = qkv[:, :nq].view(n, model.H_q, model.d_h)
    k = qkv[:, nq:nq + nk].view(n, model.H_kv, model.d_h)
    v = qkv[:, nq + nk:].view(n, model.H_kv, model.d_h)
    half = model.d_h // 2
    theta = model.rope_base ** (-torch.arange(half, dtype=torch.float64) * 2 / model.d_h)
    rot = torch.polar(torch.ones(n, half, dtype=torch.float64),
                      torch.as_tensor(pos, dtype=torch.float64)[:, None] * theta)[:, None, :]
    def rope(a):
        z = torch.complex(a[..., :half], a[..., half:]) * rot
        return torch.cat([z.real, z.imag], dim=-1)
    q, k = rope(q), rope(k)
    kb = k.float().to(torch.bfloat16)
    vb = v.float().to(torch.bfloat16)
    o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], kb.double().transpose(0, 1)[None],
                                       vb.double().transpose(0, 1)[None], is_causal=True,
                                       enable_gqa=True)[0].transpose(0, 1).reshape(n, -1)
    y = x + F.linear(o, t("w_o"))
    m = F.rms_norm(y, (model.d,), t("w_post_norm"), model.rms_eps)
    z = y + F.linear(F.silu(F.linear(m, t("w_gate"))) * F.linear(m, t("w_up")), t("w_down"))
    return z.numpy(), kb.view(torch.int16).numpy().view(np.uint16), vb.view(torch.int16).numpy().view(np.uint16)


@pytest.mark.parametrize("model", [SMALL, replace(SMALL, H_kv=4, qkv_bias=False),
                                   replace(SMALL, H_q=8, H_kv=1, d=128)])
def test_dense_layer_vs_torch_library(model):
    w = _weights(model, seed=3)
    # larger projections than the default recipe so that attention is peaked
    xb = _x_bits(40, model.d, 4)
    pos = np.arange(40) + 5
    z, Kb, Vb = fixture.dense_layer(bf16.bits_to_f64(xb), pos, w, model)
    zt, Kt, Vt = _torch_layer(xb, pos, w, model)
    assert (Kb == Kt).mean() > 0.999 and (Vb == Vt).mean() > 0.999
    assert np.abs(z - zt).max() < 1e-4


def test_recompute_all_equals_dense_layer():
    """Recomputing every token (here also the prefix) over an arbitrary cache
    is ordinary causal prefill."""
    model = SMALL
    w = _weights(model, seed=5)
    n = 48
    xb = _x_bits(n, model.d, 6)
    z, Kb, Vb = fixture.dense_layer(bf16.bits_to_f64(xb), np.arange(n), w, model)
    junk = np.random.default_rng(0).integers(0, 2 ** 15, size=Kb.shape).astype(np.uint16)
    r = layer.recompute_layer(xb, np.arange(n), junk, junk.copy(), np.arange(n), w, model)
    assert np.array_equal(r.K_bits, Kb) and np.array_equal(r.V_bits, Vb)
    assert np.abs(r.out - z).max() < 1e-10
    assert np.allclose(r.row_sums, 1.0, atol=1e-12)


def test_recompute_nothing_is_plain_concatenation():
    """idx = the query tail only: the chunk part of the cache must stay bit for
    bit what it was, and the query rows attend over stale cache + themselves."""
    model = SMALL
    w = _weights(model, seed=7)
    P, T, Q = 4, 30, 6
    n = P + T + Q
    xl, xg = _x_bits(n, model.d, 8), _x_bits(n, model.d, 9)
    Ks, Vs = fixture.stale_cache_one_layer(xl, w, model)
    Ks[P + T:], Vs[P + T:] = 0, 0
    idx = np.arange(P + T, n)
    r = layer.recompute_layer(xg, idx, Ks, Vs, idx, w, model)
    assert np.array_equal(r.K_bits[:P + T], Ks[:P + T]) and np.array_equal(r.V_bits[:P + T], Vs[:P + T])
    changed = np.nonzero((r.K_bits != Ks).any(axis=(1, 2)))[0]
    assert set(changed.tolist()) <= set(idx.tolist())
    # independent: torch SDPA of the Q fresh queries over [stale ; fresh] keys with an explicit mask
    q = torch.from_numpy(r.q_rot).transpose(0, 1)[None]                       # [1,H_q,Q,d_h]
    K = torch.from_numpy(bf16.bits_to_f64(r.K_bits)).transpose(0, 1)[None]
    V = torch.from_numpy(bf16.bits_to_f64(r.V_bits)).transpose(0, 1)[None]
    mask = torch.arange(n)[None, :] <= torch.from_numpy(idx)[:, None]
    o = F.scaled_dot_product_attention(q, K, V, attn_mask=mask, enable_gqa=True)[0]
    assert np.allclose(o.transpose(0, 1).reshape(Q, -1).numpy(), r.attn_out, atol=1e-12)


def test_scatter_positions_and_causality():
    model = SMALL
    w = _weights(model, seed=10)
    n = 64
    xl, xg = _x_bits(n, model.d, 11), _x_bits(n, model.d, 12)
    Ks, Vs = fixture.stale_cache_one_layer(xl, w, model)
    idx = np.array([5, 6, 7, 20, 21, 40, 41, 42, 43, 60, 61, 62, 63])
    r = layer.recompute_layer(xg, idx, Ks, Vs, idx, w, model)
    untouched = np.setdiff1d(np.arange(n), idx)
    assert np.array_equal(r.K_bits[untouched], Ks[untouched])
    assert np.array_equal(r.V_bits[idx], bf16.f64_to_bits(r.v_new))
    assert np.allclose(r.row_sums, 1.0, atol=1e-12)
    # dropping later tokens from the set leaves earlier rows unchanged
    r2 = layer.recompute_layer(xg, idx[:5], Ks, Vs, idx[:5], w, model)
    assert np.allclose(r2.out, r.out[:5], atol=1e-12)
    # a row's attention sees fresh K/V of earlier selected tokens, not stale ones
    r3 = layer.recompute_layer(xg, idx[3:], Ks, Vs, idx[3:], w, model)
    assert np.abs(r3.out[0] - r.out[3]).max() > 1e-6
    # gather_idx=None means hidden is already compact
    r4 = layer.recompute_layer(xg[idx], None, Ks, Vs, idx, w, model)
    assert np.allclose(r4.out, r.out, atol=1e-12)
    # rows= evaluates a subset, identically
    r5 = layer.recompute_layer(xg, idx, Ks, Vs, idx, w, model, rows=[2, 9])
    assert np.allclose(r5.out, r.out[[2, 9]], atol=1e-12)


def test_attend_row_single_key_and_uniform():
    # one visible key: output is that key's value whatever the query
    K = np.random.default_rng(0).standard_normal((3, 2, 8))
    V = np.random.default_rng(1).standard_normal((3, 2, 8))
    q = np.random.default_rng(2).standard_normal((4, 8))
    o, p = layer.attend_row(q, K, V, 0, 2)
    assert np.allclose(o, np.repeat(V[0], 2, axis=0)) and np.allclose(p, 1.0)
    # zero query: uniform weights -> mean of visible values; heads h map to kv head h // g
    o, p = layer.attend_row(np.zeros((4, 8)), K, V, 2, 2)
    assert np.allclose(p, 1 / 3) and np.allclose(o[1], V[:, 0].mean(axis=0)) \
        and np.allclose(o[2], V[:, 1].mean(axis=0))
    # 1/sqrt(d_h) scaling: q = k = e_0 * s gives logit s^2/sqrt(8) on that key
    K2 = np.zeros((2, 1, 8)); K2[1, 0, 0] = 3.0
    q2 = np.zeros((1, 8)); q2[0, 0] = 3.0
    _, p = layer.attend_row(q2, K2, np.zeros((2, 1, 8)), 1, 1)
    assert abs(p[0, 1] / p[0, 0] - math.exp(9 / math.sqrt(8))) < 1e-9


# ---------------------------------------------------------------- Section 4.1 assembly + stack end points
def test_concat_positions_and_single_prefix():
    model = SMALL
    ws = [_weights(model, seed=13)]
    P, lens, Q = 3, (5, 7, 4), 2
    n = P + sum(lens) + Q
    xb = _x_bits(n, model.d, 14)
    per = fixture.chunk_caches(xb, P, lens, ws, model)
    Kg, Vg = fixture.concat_caches(per, P, lens, Q, model, 1)
    assert Kg[0].shape == (n, model.H_kv, model.d_h)
    assert np.array_equal(Kg[0][:P], per[0][0][0][:P])             # one prefix copy, from chunk 0
    assert not Kg[0][-Q:].any()
    # layer-0 keys depend on the token alone, so re-numbered keys must agree with
    # keys computed directly at global positions (up to the second bf16 rounding)
    Kd, Vd = fixture.stale_cache_one_layer(xb, ws[0], model)
    a, b = bf16.bits_to_f64(Kg[0][:-Q]), bf16.bits_to_f64(Kd[:-Q])
    assert np.abs(a - b).max() <= 2.0 ** -7 * np.abs(b).max()
    assert np.array_equal(Vg[0][:-Q], Vd[:-Q])


@pytest.fixture(scope="module")
def two_layer():
    model = replace(SMALL, n_layers=2)
    ws = [_weights(model, seed=15, layer_id=l) for l in range(2)]
    P, lens, Q = 4, (12, 9, 15), 5
    n = P + sum(lens) + Q
    xb = _x_bits(n, model.d, 16)
    Ks, Vs = fixture.stale_caches(xb, P, lens, Q, ws, model)
    full_h, Kf, Vf = fixture.full_prefill(xb, ws, model)
    return model, ws, P, lens, Q, n, xb, Ks, Vs, full_h, Kf, Vf


def test_two_layer_recompute_everything_equals_full_prefill(two_layer):
    model, ws, P, lens, Q, n, xb, Ks, Vs, full_h, Kf, Vf = two_layer
    # the stale layer-1 cache really is stale (chunks never saw each other)
    assert (Ks[1][P + lens[0]:n - Q] != Kf[1][P + lens[0]:n - Q]).mean() > 0.5
    idx = np.arange(P, n)
    res = fixture.selective_prefill(xb, Ks, Vs, idx, ws, model)
    for l in range(2):
        assert (res[l].K_bits == Kf[l]).mean() > 0.999 and (res[l].V_bits == Vf[l]).mean() > 0.999
    a, b = bf16.bits_to_f64(res[1].out_bits), bf16.bits_to_f64(full_h[P:])
    assert (res[1].out_bits == full_h[P:]).mean() > 0.995
    assert np.abs(a - b).max() <= 2.0 ** -7 * np.abs(b).max()


def test_two_layer_recompute_nothing_is_direct_reuse(two_layer):
    model, ws, P, lens, Q, n, xb, Ks, Vs, full_h, Kf, Vf = two_layer
    idx = np.arange(n - Q, n)
    res = fixture.selective_prefill(xb, Ks, Vs, idx, ws, model)
    for l in range(2):
        assert np.array_equal(res[l].K_bits[:n - Q], Ks[l][:n - Q])
        assert np.array_equal(res[l].V_bits[:n - Q], Vs[l][:n - Q])
    # and it differs from full attention (that is the quality gap the method closes)
    assert np.abs(bf16.bits_to_f64(res[1].out_bits) - bf16.bits_to_f64(full_h[n - Q:])).max() > 1e-3


def test_partial_recompute_moves_towards_full(two_layer):
    model, ws, P, lens, Q, n, xb, Ks, Vs, full_h, Kf, Vf = two_layer
    T = sum(lens)
    def err(idx):
        res = fixture.selective_prefill(xb, Ks, Vs, idx, ws, model)
        K1 = bf16.bits_to_f64(res[1].K_bits)[P:n - Q]
        return np.abs(K1 - bf16.bits_to_f64(Kf[1])[P:n - Q]).mean()
    tail = np.arange(n - Q, n)
    e0 = err(tail)
    e_half = err(np.concatenate([np.arange(P, P + T // 2), tail]))
    e_all = err(np.arange(P, n))
    assert e_all < 1e-4 < e_half < e0


def test_tiny_config_fixture_shapes():
    wl = CONFIGS["C1"]
    w = gen.layer_weights(wl.model, 0, wl.seed)
    xl, xg = gen.hidden_pair(wl)
    assert xl.shape == (wl.N, wl.model.d) and (xl[:wl.P] == xg[:wl.P]).all()
    assert (xl[wl.P:wl.P + wl.T] != xg[wl.P:wl.P + wl.T]).mean() > 0.9
    Ks, Vs = fixture.stale_cache_one_layer(xl, w, wl.model)
    idx = gen.exact_ratio_idx(wl, 2000)
    assert len(idx) == 204 + wl.Q and (np.diff(idx) > 0).all()
    r = layer.recompute_layer(xg, idx, Ks, Vs, idx, w, wl.model, rows=[0, 100, len(idx) - 1])
    assert np.allclose(r.row_sums, 1.0, atol=1e-12) and np.isfinite(r.out).all()


def test_kv_only_projection_equals_full_projection():
    """kv_rows / q_for_rows_only are the same numbers as the full projection."""
    model = ModelShape(128, 4, 2, 32, 64, 1e4, 1e-5, True, 1)
    w = gen.layer_weights(model, 0, seed=31)
    r = np.random.default_rng(3)
    N = 40
    xb = gen.f32_to_bf16_bits(r.standard_normal((N, model.d)).astype(np.float32))
    Kb = gen.f32_to_bf16_bits(r.standard_normal((N, model.H_kv, model.d_h)).astype(np.float32))
    Vb = gen.f32_to_bf16_bits(r.standard_normal((N, model.H_kv, model.d_h)).astype(np.float32))
    idx = np.array([2, 3, 9, 17, 18, 39])
    rows = np.array([1, 4, 5])
    full = layer.recompute_layer(xb, idx, Kb, Vb, idx, w, model, rows=rows)
    part = layer.recompute_layer(xb, idx, Kb, Vb, idx, w, model, rows=rows, q_for_rows_only=True)
    assert np.array_equal(full.K_bits, part.K_bits) and np.array_equal(full.V_bits, part.V_bits)
    np.testing.assert_allclose(part.k_new, full.k_new, rtol=0, atol=1e-12)
    np.testing.assert_allclose(part.out, full.out, rtol=0, atol=1e-12)
    np.testing.assert_allclose(part.q_rot[rows], full.q_rot[rows], rtol=0, atol=1e-12)
