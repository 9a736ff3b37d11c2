"""GPU parity of cc_recompute_layer and its stages against the oracle.

Tolerances (bf16 inputs, fp32 accumulation, fp64 oracle): layer outputs and
updated K/V rows max abs <= 2e-2 and mean abs <= 2e-3; scatter positions and
untouched cache rows bit-exact.
"""
from dataclasses import replace

import numpy as np
import pytest
import torch

import paper_2510_10129_amd as cc
from paper_2510_10129_amd import _lib
from oracle import bf16 as obf
from oracle import fixture, layer
from workloads import CONFIGS, ModelShape, gen

from _gpu_util import DEV, bits_f64, dev_bf16, dev_i32, dev_weights, err_stats, host_bits

pytestmark = pytest.mark.gpu
MAX_ABS, MEAN_ABS = 2e-2, 2e-3


def _ctx(model, N, M):
    return cc.Context.for_model(model, N_cap=N, M_cap=max(M, 1), T_cap=1024)


def _x_bits(n, d, seed, scale=1.0):
    r = np.random.default_rng(seed)
    return gen.f32_to_bf16_bits((r.standard_normal((n, d)) * scale).astype(np.float32))


def _run_layer(model, xg_bits, gather, Ks, Vs, idx, w, rows=None, flags=_lib.FLAG_CHECK_IDX):
    """Runs the HIP layer and the oracle on the same inputs; returns both."""
    N, M = Ks.shape[0], len(idx)
    ctx = _ctx(model, N, M)
    Kd, Vd = dev_bf16(Ks), dev_bf16(Vs)
    hid = dev_bf16(xg_bits)
    out = torch.full((max(M, 1), model.d), float("nan"), dtype=torch.bfloat16, device=DEV)
    ctx.recompute_layer(hid, None if gather is None else dev_i32(gather), cc.KVLayer(Kd, Vd),
                        dev_i32(idx), M, dev_weights(w), out, flags)
    torch.cuda.synchronize()
    ref = layer.recompute_layer(xg_bits, gather, Ks, Vs, idx, w, model, rows=rows)
    got = dict(out=host_bits(out)[:M], K=host_bits(Kd), V=host_bits(Vd))
    ctx.close()
    return got, ref


def _assert_layer(got, ref, Ks, Vs, idx, tag="", kv_scale=1.0):
    idx = np.asarray(idx)
    N = Ks.shape[0]
    untouched = np.setdiff1d(np.arange(N), idx)
    # scatter positions: every row outside idx keeps its bits
    assert np.array_equal(got["K"][untouched], Ks[untouched]), tag
    assert np.array_equal(got["V"][untouched], Vs[untouched]), tag
    # fresh rows against the oracle's unrounded values
    for name, fresh in (("K", ref.k_new), ("V", ref.v_new)):
        mx, mn = err_stats(bits_f64(got[name][idx]), fresh)
        assert mx <= MAX_ABS * kv_scale and mn <= MEAN_ABS * kv_scale, (tag, name, mx, mn)
    mx, mn = err_stats(bits_f64(got["out"][ref.rows]), ref.out)
    print(f"{tag}: out max {mx:.2e} mean {mn:.2e}")
    assert np.isfinite(bits_f64(got["out"])).all(), tag
    # stress cases with amplified weights have outputs larger than the recipe's
    # O(1); bf16 spacing grows with the value, so the bound follows the rms there
    os_ = 1.0 if kv_scale == 1.0 else max(1.0, float(np.sqrt(np.mean(ref.out ** 2))))
    assert mx <= MAX_ABS * os_ and mn <= MEAN_ABS * os_, (tag, mx, mn, os_)


def test_tiny_config_full_parity():
    wl = CONFIGS["C1"]
    w = gen.layer_weights(wl.model, 0, wl.seed)
    xl, xg = gen.hidden_pair(wl)
    Ks, Vs = fixture.stale_cache_one_layer(xl, w, wl.model)
    Ks[wl.P + wl.T:], Vs[wl.P + wl.T:] = 0, 0
    from oracle import select as osel
    idx = osel.select(gen.aux_attention(wl), 2000, wl.window, wl.tau, True, wl.P, wl.Q)
    got, ref = _run_layer(wl.model, xg, idx, Ks, Vs, idx, w)
    _assert_layer(got, ref, Ks, Vs, idx, "C1")
    # the stale rows that were recomputed really changed
    assert (got["K"][idx[:-wl.Q]] != Ks[idx[:-wl.Q]]).mean() > 0.5


SHAPES = [
    # (model, N, idx builder) - head dims, group sizes, bias, ragged sizes
    (ModelShape(128, 4, 2, 64, 192, 1e4, 1e-5, False, 1), 300, "runs"),
    (ModelShape(256, 2, 2, 128, 320, 5e5, 1e-5, True, 1), 257, "all"),
    (ModelShape(448, 7, 1, 64, 128, 1e6, 1e-6, True, 1), 200, "runs"),
    (ModelShape(1024, 8, 1, 128, 256, 5e5, 1e-5, False, 1), 333, "tail"),
    (ModelShape(192, 3, 1, 64, 64, 1e4, 1e-5, False, 1), 131, "single"),
    (ModelShape(2048, 32, 1, 64, 128, 1e4, 1e-5, False, 1), 100, "runs"),
]


def _shape_idx(kind, N, rng):
    if kind == "all":
        return np.arange(N)
    if kind == "tail":
        return np.arange(N - 9, N)
    if kind == "single":
        return np.array([77])
    marks = np.zeros(N, bool)
    for s in rng.integers(1, N - 10, size=N // 12):
        marks[s:s + int(rng.integers(1, 9))] = True
    marks[N - 5:] = True
    return np.nonzero(marks)[0]


@pytest.mark.parametrize("model,N,kind", SHAPES)
def test_shapes_and_edge_cases(model, N, kind):
    rng = np.random.default_rng(N)
    w = gen.layer_weights(model, 0, seed=N)
    # bigger projections than the default recipe: peaked attention, every key matters
    wq = gen.bf16_to_f32(w["w_qkv"]).copy()
    n_qk = (model.H_q + model.H_kv) * model.d_h            # q and k rows only; v stays O(1)
    wq[:n_qk] *= 3.0
    w["w_qkv"] = gen.f32_to_bf16_bits(wq)
    xl, xg = _x_bits(N, model.d, 1), _x_bits(N, model.d, 2)
    Ks, Vs = fixture.stale_cache_one_layer(xl, w, model)
    idx = _shape_idx(kind, N, rng)
    got, ref = _run_layer(model, xg, idx, Ks, Vs, idx, w)
    # K/V are three times the recipe's size here and bf16 spacing grows with them
    _assert_layer(got, ref, Ks, Vs, idx, f"{kind} d={model.d} g={model.g} d_h={model.d_h}", kv_scale=3.0)


@pytest.mark.parametrize("model,N,kind", SHAPES)
def test_shapes_and_edge_cases_recipe_weights_strict_bound(model, N, kind):
    """The same shapes and index sets (a tail, a single row, every row, groups of 7 and of 32
    query heads, head dims 64 and 128, bias) with the weights of the input recipe as they are:
    the stated bound, 2e-2 / 2e-3, with no allowance."""
    rng = np.random.default_rng(N)
    w = gen.layer_weights(model, 0, seed=N)
    xl, xg = _x_bits(N, model.d, 1), _x_bits(N, model.d, 2)
    Ks, Vs = fixture.stale_cache_one_layer(xl, w, model)
    got, ref = _run_layer(model, xg, (idx := _shape_idx(kind, N, rng)), Ks, Vs, idx, w)
    _assert_layer(got, ref, Ks, Vs, idx, f"strict {kind} d={model.d} g={model.g} d_h={model.d_h}")


@pytest.mark.parametrize("seed", range(10))
def test_random_small_layers(seed):
    """Seeded random layer shapes and token sets (head dims, group sizes 1..8, widths that take the
    ring and the staged K loop, context lengths across several key tiles, sparse and dense idx):
    the whole layer against the oracle with the launchers' own choices."""
    rng = np.random.default_rng(1000 + seed)
    d_h = int(rng.choice([64, 128]))
    H_kv = int(rng.choice([1, 2, 4]))
    g = int(rng.choice([1, 2, 3, 4, 7, 8]))
    d = 64 * int(rng.integers(2, 17))
    f = 64 * int(rng.integers(1, 17))
    model = ModelShape(d, g * H_kv, H_kv, d_h, f, float(rng.choice([1e4, 5e5, 1e6])),
                       float(rng.choice([1e-5, 1e-6])), bool(rng.integers(0, 2)), 1)
    N = int(rng.integers(20, 1200))
    marks = rng.random(N) < rng.uniform(0.05, 0.9)
    marks[N - 1] = True
    idx = np.nonzero(marks)[0]
    w = gen.layer_weights(model, 0, seed=2000 + seed)
    xl, xg = _x_bits(N, d, 3 * seed + 1), _x_bits(N, d, 3 * seed + 2)
    Ks, Vs = fixture.stale_cache_one_layer(xl, w, model)
    rows = None if len(idx) <= 96 else np.unique(np.concatenate([[0, len(idx) - 1], rng.choice(len(idx), 64, replace=False)]))
    got, ref = _run_layer(model, xg, idx, Ks, Vs, idx, w, rows=rows)
    _assert_layer(got, ref, Ks, Vs, idx, f"seed {seed}: d={d} f={f} {g * H_kv}q/{H_kv}kv d_h={d_h} N={N} M={len(idx)}")


def test_layer_results_are_bit_reproducible():
    """Nothing in the layer adds in a run-dependent order: three runs of one layer on the same
    inputs (ring loop with the 256x256 tile, split attention) give the same bits."""
    model = ModelShape(512, 8, 2, 64, 1024, 1e4, 1e-5, True, 1)
    N = 700
    rng = np.random.default_rng(3)
    marks = rng.random(N) < 0.6
    marks[N - 1] = True
    idx = np.nonzero(marks)[0]
    M = len(idx)
    w = gen.layer_weights(model, 0, seed=8)
    xl, xg = _x_bits(N, model.d, 31), _x_bits(N, model.d, 32)
    Ks, Vs = fixture.stale_cache_one_layer(xl, w, model)
    ctx = _ctx(model, N, M)
    dw, hid, di = dev_weights(w), dev_bf16(xg), dev_i32(idx)
    runs = []
    for _ in range(3):
        Kd, Vd = dev_bf16(Ks), dev_bf16(Vs)
        out = torch.empty((M, model.d), dtype=torch.bfloat16, device=DEV)
        ctx.recompute_layer(hid, di, cc.KVLayer(Kd, Vd), di, M, dw, out, 0)
        torch.cuda.synchronize()
        runs.append((host_bits(out).copy(), host_bits(Kd).copy(), host_bits(Vd).copy()))
    for r in runs[1:]:
        for a, b in zip(runs[0], r):
            assert np.array_equal(a, b)
    ctx.close()


def test_compact_hidden_and_zero_rows():
    model = SHAPES[0][0]
    N = 150
    w = gen.layer_weights(model, 0, seed=9)
    xl, xg = _x_bits(N, model.d, 3), _x_bits(N, model.d, 4)
    Ks, Vs = fixture.stale_cache_one_layer(xl, w, model)
    idx = np.array([3, 4, 5, 60, 61, 62, 63, 149])
    got, ref = _run_layer(model, xg[idx], None, Ks, Vs, idx, w)      # hidden already compact
    _assert_layer(got, ref, Ks, Vs, idx, "compact")
    # M = 0: nothing changes, no error
    ctx = _ctx(model, N, 4)
    Kd, Vd = dev_bf16(Ks), dev_bf16(Vs)
    out = torch.zeros((1, model.d), dtype=torch.bfloat16, device=DEV)
    ctx.recompute_layer(dev_bf16(xg), None, cc.KVLayer(Kd, Vd), dev_i32([0]), 0, dev_weights(w), out)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(Kd), Ks) and np.array_equal(host_bits(Vd), Vs)
    ctx.close()


def test_strided_cache_view():
    """K and V as slices of one [N, 2, H_kv, d_h] allocation (token stride 2*H_kv*d_h)."""
    model = SHAPES[0][0]
    N = 120
    w = gen.layer_weights(model, 0, seed=11)
    xl, xg = _x_bits(N, model.d, 5), _x_bits(N, model.d, 6)
    Ks, Vs = fixture.stale_cache_one_layer(xl, w, model)
    idx = np.array([10, 11, 12, 13, 50, 51, 118, 119])
    both = torch.stack([dev_bf16(Ks), dev_bf16(Vs)], dim=1).contiguous()
    Kd, Vd = both[:, 0], both[:, 1]
    ctx = _ctx(model, N, len(idx))
    out = torch.empty((len(idx), model.d), dtype=torch.bfloat16, device=DEV)
    ctx.recompute_layer(dev_bf16(xg), dev_i32(idx), cc.KVLayer(Kd, Vd), dev_i32(idx), len(idx),
                        dev_weights(w), out, _lib.FLAG_CHECK_IDX)
    torch.cuda.synchronize()
    ref = layer.recompute_layer(xg, idx, Ks, Vs, idx, w, model)
    got = dict(out=host_bits(out), K=host_bits(Kd), V=host_bits(Vd))
    _assert_layer(got, ref, Ks, Vs, idx, "strided")
    ctx.close()


def test_idx_check_and_argument_errors():
    model = SHAPES[0][0]
    N = 64
    w = gen.layer_weights(model, 0, seed=12)
    x = _x_bits(N, model.d, 7)
    Ks, Vs = fixture.stale_cache_one_layer(x, w, model)
    ctx = _ctx(model, N, 8)
    Kd, Vd = dev_bf16(Ks), dev_bf16(Vs)
    out = torch.empty((8, model.d), dtype=torch.bfloat16, device=DEV)
    args = lambda idx, M: (dev_bf16(x), dev_i32(idx), cc.KVLayer(Kd, Vd), dev_i32(idx), M, dev_weights(w), out)
    for bad in ([5, 5, 6], [7, 6, 8], [1, 2, 64], [-1, 2, 3]):
        with pytest.raises(cc.CacheClipError) as e:
            ctx.recompute_layer(*args(bad, 3), _lib.FLAG_CHECK_IDX)
        assert e.value.status == _lib.CC_ERR_IDX
    with pytest.raises(cc.CacheClipError) as e:
        ctx.recompute_layer(*args(list(range(9)), 9))
    assert e.value.status == _lib.CC_ERR_WORKSPACE
    with pytest.raises(cc.CacheClipError) as e:
        ctx.recompute_layer(*args([1], -1))
    assert e.value.status == _lib.CC_ERR_SHAPE
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(Kd), Ks)          # failed calls wrote nothing
    ctx.close()


# ------------------------------------------------------------ single stages
@pytest.mark.parametrize("splits", ["", "1", "2", "3", "8"])
def test_stage_attention_peaked_random(splits):
    """The attention kernel alone, on q/K/V drawn directly so that the softmax is
    sharply peaked and the causal boundary matters; with the launcher's own choice of key
    splits and with 1, 2, 3 and 8 forced (cc_debug_set_launch; more splits than key tiles
    leave empty parts)."""
    for (H_q, H_kv, d_h, N, seed) in ((8, 2, 128, 700, 0), (4, 4, 64, 333, 1), (7, 1, 128, 190, 2),
                                      (16, 2, 64, 1000, 3)):
        rng = np.random.default_rng(seed)
        model = ModelShape(H_q * d_h, H_q, H_kv, d_h, 64, 1e4, 1e-5, False, 1)
        marks = rng.random(N) < 0.3
        marks[0] = True
        marks[N - 1] = True
        idx = np.nonzero(marks)[0]
        M = len(idx)
        qb = gen.f32_to_bf16_bits((rng.standard_normal((M, H_q, d_h)) * 2.5).astype(np.float32))
        Kb = gen.f32_to_bf16_bits(rng.standard_normal((N, H_kv, d_h)).astype(np.float32))
        Vb = gen.f32_to_bf16_bits(rng.standard_normal((N, H_kv, d_h)).astype(np.float32))
        ctx = _ctx(model, N, M)
        ctx.debug_set_launch(attn_splits=int(splits) if splits else 0)
        o = torch.empty((M, H_q * d_h), dtype=torch.bfloat16, device=DEV)
        ctx.step_sparse_attention(dev_bf16(qb).view(M, -1), M, dev_i32(idx),
                                  cc.KVLayer(dev_bf16(Kb), dev_bf16(Vb)), o, _lib.FLAG_CHECK_IDX)
        torch.cuda.synchronize()
        qf, Kf, Vf = obf.bits_to_f64(qb), obf.bits_to_f64(Kb), obf.bits_to_f64(Vb)
        ref = np.stack([layer.attend_row(qf[i], Kf, Vf, int(idx[i]), H_q // H_kv)[0].reshape(-1)
                        for i in range(M)])
        mx, mn = err_stats(bits_f64(host_bits(o)), ref)
        print(f"attention H_q={H_q} H_kv={H_kv} d_h={d_h}: max {mx:.2e} mean {mn:.2e}")
        assert mx <= MAX_ABS and mn <= MEAN_ABS
        ctx.close()


@pytest.mark.parametrize("N", [1, 2, 63, 64, 65, 127, 128, 129, 192, 193, 257, 320])
def test_stage_attention_key_tile_boundaries(N):
    """Cache lengths around the 64-key tile and the three-stage load pipeline (1, 2, 3, 4+
    tiles), with every row recomputed and with a handful of rows (so that one of the two wave
    groups of a workgroup, or most of its waves, own no column)."""
    for (H_q, H_kv, d_h, picks) in ((4, 2, 128, "all"), (8, 1, 64, "few"), (2, 2, 128, "few")):
        rng = np.random.default_rng(N * 7 + H_q)
        model = ModelShape(H_q * d_h, H_q, H_kv, d_h, 64, 1e4, 1e-5, False, 1)
        idx = np.arange(N) if picks == "all" else np.unique(np.r_[0, rng.integers(0, N, size=3), N - 1])
        M = len(idx)
        qb = gen.f32_to_bf16_bits((rng.standard_normal((M, H_q, d_h)) * 2.0).astype(np.float32))
        Kb = gen.f32_to_bf16_bits(rng.standard_normal((N, H_kv, d_h)).astype(np.float32))
        Vb = gen.f32_to_bf16_bits(rng.standard_normal((N, H_kv, d_h)).astype(np.float32))
        ctx = _ctx(model, N, M)
        o = torch.full((M, H_q * d_h), float("nan"), dtype=torch.bfloat16, device=DEV)
        ctx.step_sparse_attention(dev_bf16(qb).view(M, -1), M, dev_i32(idx),
                                  cc.KVLayer(dev_bf16(Kb), dev_bf16(Vb)), o, _lib.FLAG_CHECK_IDX)
        torch.cuda.synchronize()
        qf, Kf, Vf = obf.bits_to_f64(qb), obf.bits_to_f64(Kb), obf.bits_to_f64(Vb)
        ref = np.stack([layer.attend_row(qf[i], Kf, Vf, int(idx[i]), H_q // H_kv)[0].reshape(-1)
                        for i in range(M)])
        mx, mn = err_stats(bits_f64(host_bits(o)), ref)
        assert mx <= MAX_ABS and mn <= MEAN_ABS, (N, H_q, H_kv, d_h, picks, mx, mn)
        ctx.close()


def test_stage_attention_many_column_blocks_long_and_short_rows():
    """Several 256-column blocks per kv head whose rows end at very different keys: within a
    block the waves stop at different tiles while the block keeps loading."""
    H_q, H_kv, d_h, N = 8, 2, 128, 1500
    rng = np.random.default_rng(5)
    model = ModelShape(H_q * d_h, H_q, H_kv, d_h, 64, 1e4, 1e-5, False, 1)
    idx = np.unique(np.r_[np.arange(0, 40), rng.integers(40, N, size=200), np.arange(N - 30, N)])
    M = len(idx)
    qb = gen.f32_to_bf16_bits((rng.standard_normal((M, H_q, d_h)) * 2.0).astype(np.float32))
    Kb = gen.f32_to_bf16_bits(rng.standard_normal((N, H_kv, d_h)).astype(np.float32))
    Vb = gen.f32_to_bf16_bits(rng.standard_normal((N, H_kv, d_h)).astype(np.float32))
    ctx = _ctx(model, N, M)
    o = torch.full((M, H_q * d_h), float("nan"), dtype=torch.bfloat16, device=DEV)
    ctx.step_sparse_attention(dev_bf16(qb).view(M, -1), M, dev_i32(idx),
                              cc.KVLayer(dev_bf16(Kb), dev_bf16(Vb)), o, _lib.FLAG_CHECK_IDX)
    torch.cuda.synchronize()
    qf, Kf, Vf = obf.bits_to_f64(qb), obf.bits_to_f64(Kb), obf.bits_to_f64(Vb)
    rows = np.unique(np.r_[np.arange(0, 12), rng.integers(0, M, size=40), np.arange(M - 12, M)])
    ref = np.stack([layer.attend_row(qf[i], Kf, Vf, int(idx[i]), H_q // H_kv)[0].reshape(-1) for i in rows])
    mx, mn = err_stats(bits_f64(host_bits(o)[rows]), ref)
    assert np.isfinite(bits_f64(host_bits(o))).all()
    assert mx <= MAX_ABS and mn <= MEAN_ABS, (mx, mn)
    ctx.close()


@pytest.mark.parametrize("splits", [1, 2])
def test_stage_attention_score_jumps_on_both_sides_of_the_rescale_threshold(splits):
    """The kernel moves the reference point of its base-2 exponent only when a row's maximum
    grows by more than 8 (a factor 2^8); below that it keeps the old reference and accumulates
    probabilities up to 256.  Both branches by construction: queries and keys live on one
    coordinate, q = (a, 0, ..), K[j] = (b_j, 0, ..) with b_j constant over each 64-key tile (0,
    1, 2.25, 1.5, -3), so the score in base-2 units of every key of tile t is c * b_t with
    c = a * log2(e) / sqrt(d_h), exactly (one bf16 product per score).  Rows, by their c: a jump
    of 7.96 over the reference (kept), 8.03 (moved), one move then a keep, two moves, falling
    scores, and neighbours in one wave that decide differently.  V is random, so an unscaled or
    doubly scaled accumulator shows in the output."""
    H_q, H_kv, d_h = 2, 1, 128
    n_tiles = 5
    N = 64 * n_tiles + 40
    b_tile = np.array([0.0, 1.0, 2.25, 1.5, -3.0, 0.5])
    a_vals = np.array([27.75, 28.0, 58.5, 67.0, -20.0, 3.0, 27.75, 67.0, 28.0, 0.0])    # all exact in bf16
    k = np.log2(np.e) / np.sqrt(float(d_h))
    c = a_vals * k
    assert 7.9 < c[0] * 2.25 < 7.99 and 8.01 < c[1] * 2.25 < 8.1          # just under / just over, tile 2
    assert 7.3 < c[2] * 1.0 < 7.99 and c[2] * 2.25 - 0.0 > 8.01           # kept at tile 1, moved at tile 2
    assert c[3] * 1.0 > 8.01 and c[3] * 2.25 - c[3] * 1.0 > 8.01          # moved twice
    idx = np.arange(N - 20, N)                      # every row sees all five tiles and part of a sixth
    M = len(idx)
    rng = np.random.default_rng(42)
    q = np.zeros((M, H_q, d_h), np.float32)
    for i in range(M):
        for h in range(H_q):
            q[i, h, 0] = a_vals[(2 * i + h) % len(a_vals)]
    K = np.zeros((N, H_kv, d_h), np.float32)
    K[:, 0, 0] = b_tile[np.arange(N) // 64]
    K[:, 0, 1:] = rng.standard_normal((N, d_h - 1))            # q is zero there: no effect on the scores
    V = rng.standard_normal((N, H_kv, d_h)).astype(np.float32)
    qb, Kb, Vb = (gen.f32_to_bf16_bits(x) for x in (q, K, V))
    assert np.array_equal(gen.bf16_to_f32(qb), q) and np.array_equal(gen.bf16_to_f32(Kb)[:, 0, 0], K[:, 0, 0])
    model = ModelShape(H_q * d_h, H_q, H_kv, d_h, 64, 1e4, 1e-5, False, 1)
    ctx = _ctx(model, N, M)
    ctx.debug_set_launch(attn_splits=splits)
    o = torch.full((M, H_q * d_h), float("nan"), dtype=torch.bfloat16, device=DEV)
    ctx.step_sparse_attention(dev_bf16(qb).view(M, -1), M, dev_i32(idx),
                              cc.KVLayer(dev_bf16(Kb), dev_bf16(Vb)), o, _lib.FLAG_CHECK_IDX)
    torch.cuda.synchronize()
    qf, Kf, Vf = obf.bits_to_f64(qb), obf.bits_to_f64(Kb), obf.bits_to_f64(Vb)
    ref = np.stack([layer.attend_row(qf[i], Kf, Vf, int(idx[i]), H_q // H_kv)[0].reshape(-1) for i in range(M)])
    got = bits_f64(host_bits(o))
    mx, mn = err_stats(got, ref)
    print(f"score jumps, {splits} split(s): max {mx:.2e} mean {mn:.2e}")
    assert mx <= MAX_ABS and mn <= MEAN_ABS, (mx, mn)
    ctx.close()


def test_stage_attention_never_reads_past_the_valid_slots():
    """The cache allocation is longer than kv->N and holds NaN beyond it: the last key tile is
    cut at N (loads are clamped to slot N-1), so nothing of it reaches the output."""
    H_q, H_kv, d_h, N, extra = 4, 2, 128, 150, 64
    rng = np.random.default_rng(9)
    model = ModelShape(H_q * d_h, H_q, H_kv, d_h, 64, 1e4, 1e-5, False, 1)
    idx = np.array([0, 5, 63, 64, 100, 149])
    M = len(idx)
    qb = gen.f32_to_bf16_bits(rng.standard_normal((M, H_q, d_h)).astype(np.float32))
    Kb = gen.f32_to_bf16_bits(rng.standard_normal((N, H_kv, d_h)).astype(np.float32))
    Vb = gen.f32_to_bf16_bits(rng.standard_normal((N, H_kv, d_h)).astype(np.float32))
    nan = np.full((extra, H_kv, d_h), 0x7FC0, np.uint16)
    Kd, Vd = dev_bf16(np.concatenate([Kb, nan])), dev_bf16(np.concatenate([Vb, nan]))
    ctx = _ctx(model, N, M)
    o = torch.full((M, H_q * d_h), float("nan"), dtype=torch.bfloat16, device=DEV)
    ctx.step_sparse_attention(dev_bf16(qb).view(M, -1), M, dev_i32(idx), cc.KVLayer(Kd[:N], Vd[:N]), o,
                              _lib.FLAG_CHECK_IDX)
    torch.cuda.synchronize()
    qf, Kf, Vf = obf.bits_to_f64(qb), obf.bits_to_f64(Kb), obf.bits_to_f64(Vb)
    ref = np.stack([layer.attend_row(qf[i], Kf, Vf, int(idx[i]), H_q // H_kv)[0].reshape(-1) for i in range(M)])
    got = bits_f64(host_bits(o))
    assert np.isfinite(got).all()
    mx, mn = err_stats(got, ref)
    assert mx <= MAX_ABS and mn <= MEAN_ABS, (mx, mn)
    ctx.close()


@pytest.mark.parametrize("tile,splitk,mfma", [("", "", ""), ("b", "", ""), ("b", "", "32"), ("m", "", ""), ("h", "", ""),
                                              ("s", "", ""), ("bt", "", ""), ("st", "", ""), ("", "2", ""), ("", "3", ""),
                                              ("", "4", ""), ("m", "2", ""), ("b", "2", "32"), ("m", "", "32"), ("m", "2", "32"), ("h", "", "32"), ("s", "", "32")])
def test_stage_projections_against_oracle_pieces(tile, splitk, mfma):
    """Every projection against the oracle's pieces, by default, with each GEMM tile shape and K
    loop forced (the 256x256 tile with its 16x16x32 loop and with the 32x32x16 one), and with 2, 3
    and 4 shares of K (3 divides only the down projection's K here, 4 leaves a share of exactly one
    ring of slices); forced through cc_debug_set_launch."""
    model = ModelShape(512, 8, 2, 64, 768, 1e4, 1e-5, True, 1)
    N, M = 500, 203
    rng = np.random.default_rng(5)
    w = gen.layer_weights(model, 0, seed=21)
    xb = _x_bits(N, model.d, 8)
    idx = np.sort(rng.choice(N, size=M, replace=False))
    ctx = _ctx(model, N, M)
    ctx.debug_set_launch(gemm_tile=tile[:1], gemm_staged=tile.endswith("t"), gemm_mfma32=mfma == "32",
                         gemm_splitk=int(splitk) if splitk else 0)
    dw = dev_weights(w)
    hid = dev_bf16(xb)
    # R1 gather + RMSNorm
    xn = torch.empty((M, model.d), dtype=torch.bfloat16, device=DEV)
    ctx.step_gather_rmsnorm(hid, dev_i32(idx), M, dw.w_in_norm, xn)
    xf = obf.bits_to_f64(xb[idx])
    n_ref = layer.rmsnorm(xf, obf.bits_to_f64(w["w_in_norm"]), model.rms_eps)
    mx, _ = err_stats(bits_f64(host_bits(xn)), n_ref)
    assert mx <= 2.0 ** -8 * np.abs(n_ref).max()
    # R2-R4 QKV + RoPE + scatter
    Ks = np.zeros((N, model.H_kv, model.d_h), np.uint16)
    Kd, Vd = dev_bf16(Ks), dev_bf16(Ks)
    q = torch.empty((M, model.H_q * model.d_h), dtype=torch.bfloat16, device=DEV)
    ctx.step_qkv_rope_scatter(xn, M, dev_i32(idx), dw.w_qkv, dw.b_qkv, cc.KVLayer(Kd, Vd), q,
                              _lib.FLAG_CHECK_IDX)
    q_ref, k_ref, v_ref = layer.qkv_rows(xf, w, model, idx)
    for got, ref in ((host_bits(q).reshape(M, model.H_q, -1), q_ref),
                     (host_bits(Kd)[idx], k_ref), (host_bits(Vd)[idx], v_ref)):
        mx, mn = err_stats(bits_f64(got), ref)
        assert mx <= MAX_ABS and mn <= MEAN_ABS, (mx, mn)
    rest = np.setdiff1d(np.arange(N), idx)
    assert not host_bits(Kd)[rest].any() and not host_bits(Vd)[rest].any()
    # R6 O projection + residual
    ob = _x_bits(M, model.H_q * model.d_h, 9, 0.5)
    y = torch.empty((M, model.d), dtype=torch.float32, device=DEV)
    ctx.step_oproj_residual(dev_bf16(ob), M, dw.w_o, hid, dev_i32(idx), y)
    y_ref = xf + obf.bits_to_f64(ob) @ obf.bits_to_f64(w["w_o"]).T
    mx, mn = err_stats(y.cpu().numpy().astype(np.float64), y_ref)
    assert mx <= 1e-4, mx                      # fp32 accumulation of exact bf16 products
    # R7 MLP
    out = torch.empty((M, model.d), dtype=torch.bfloat16, device=DEV)
    ctx.step_mlp(y, M, dw.w_post_norm, dw.w_gate, dw.w_up, dw.w_down, out)
    torch.cuda.synchronize()
    yf = y.cpu().numpy().astype(np.float64)
    m = layer.rmsnorm(yf, obf.bits_to_f64(w["w_post_norm"]), model.rms_eps)
    z = yf + (layer.silu(m @ obf.bits_to_f64(w["w_gate"]).T) * (m @ obf.bits_to_f64(w["w_up"]).T)) \
        @ obf.bits_to_f64(w["w_down"]).T
    mx, mn = err_stats(bits_f64(host_bits(out)), z)
    assert mx <= MAX_ABS and mn <= MEAN_ABS, (mx, mn)
    ctx.close()


@pytest.mark.parametrize("splitk,tile", [("2", ""), ("2", "m"), ("3", "")])
def test_stage_mlp_wide_grid_with_split_last_round(splitk, tile):
    """A gate/up grid of 258 tiles (one full round of workgroups and two tiles more): with two K
    shares forced the full round runs as one launch and the two remaining tiles as split-K with
    the finishing pass; three shares divide only the down projection's K (2 tiles, split whole)."""
    model = ModelShape(256, 4, 2, 64, 16512, 1e4, 1e-5, False, 1)
    M = 300
    rng = np.random.default_rng(11)
    w = gen.layer_weights(model, 0, seed=33)
    ctx = _ctx(model, 64, M)
    ctx.debug_set_launch(gemm_tile=tile, gemm_splitk=int(splitk))
    dw = dev_weights(w)
    y = torch.from_numpy(rng.standard_normal((M, model.d)).astype(np.float32)).to(DEV)
    out = torch.empty((M, model.d), dtype=torch.bfloat16, device=DEV)
    ctx.step_mlp(y, M, dw.w_post_norm, dw.w_gate, dw.w_up, dw.w_down, out)
    torch.cuda.synchronize()
    yf = y.cpu().numpy().astype(np.float64)
    m = layer.rmsnorm(yf, obf.bits_to_f64(w["w_post_norm"]), model.rms_eps)
    z = yf + (layer.silu(m @ obf.bits_to_f64(w["w_gate"]).T) * (m @ obf.bits_to_f64(w["w_up"]).T)) \
        @ obf.bits_to_f64(w["w_down"]).T
    mx, mn = err_stats(bits_f64(host_bits(out)), z)
    assert mx <= MAX_ABS and mn <= MEAN_ABS, (mx, mn)
    ctx.close()


# ------------------------------------------------------------ stack and full-size shapes
def test_two_layer_stack_with_real_stale_caches():
    wl = CONFIGS["C1x2"]
    model = wl.model
    ws = [gen.layer_weights(model, l, wl.seed) for l in range(2)]
    xl, _ = gen.hidden_pair(wl)
    Ks, Vs = fixture.stale_caches(xl, wl.P, wl.chunk_lens, wl.Q, ws, model)
    idx = gen.exact_ratio_idx(wl, 2000)
    M = len(idx)
    ref = fixture.selective_prefill(xl, Ks, Vs, idx, ws, model)
    ctx = _ctx(model, wl.N, M)
    didx = dev_i32(idx)
    # (a) each layer on the oracle's input for that layer: the per-layer bound holds
    # (b) chained on the device's own layer-0 output: a bf16 code that rounded the other
    #     way below rides the residual stream, so allow one output spacing on top
    h_chain, g_chain = dev_bf16(xl), didx
    for l in range(2):
        h_tf, g_tf = (dev_bf16(xl), didx) if l == 0 else (dev_bf16(ref[l - 1].out_bits), None)
        for mode, (h, g) in (("teacher-forced", (h_tf, g_tf)), ("chained", (h_chain, g_chain))):
            Kd, Vd = dev_bf16(Ks[l]), dev_bf16(Vs[l])
            out = torch.empty((M, model.d), dtype=torch.bfloat16, device=DEV)
            ctx.recompute_layer(h, g, cc.KVLayer(Kd, Vd), didx, M, dev_weights(ws[l]), out,
                                _lib.FLAG_CHECK_IDX)
            torch.cuda.synchronize()
            got = dict(out=host_bits(out), K=host_bits(Kd), V=host_bits(Vd))
            if mode == "teacher-forced":
                _assert_layer(got, ref[l], Ks[l], Vs[l], idx, f"stack layer {l}")
            else:
                mx, mn = err_stats(bits_f64(got["out"]), ref[l].out)
                print(f"stack layer {l} chained: out max {mx:.2e} mean {mn:.2e}")
                assert mx <= MAX_ABS + 2.0 ** -7 * np.abs(ref[l].out).max() and mn <= MEAN_ABS
                h_chain, g_chain = out, None
    ctx.close()


def test_eight_layer_stack_drift_at_the_4k_shape(capsys):
    """How far a stack drifts: eight Llama-3-8B-shaped layers of the 4k workload at 20 %, (a) each
    layer on the oracle's own input for that layer (teacher-forced: the per-layer bound must hold
    at every depth) and (b) chained on the device's own outputs against the oracle chained on
    its own (recorded: rounding differences ride the residual stream, so this error grows with
    depth; bounded here only against a blow-up).  Weights, hidden rows and stale caches are
    drawn on the device; every row of every layer is compared."""
    from workloads import gen_device
    n_layers = 8
    wl = CONFIGS["C2"]
    model = replace(wl.model, n_layers=n_layers)
    wl = replace(wl, model=model)
    dev = torch.device(DEV)
    idx = gen.exact_ratio_idx(wl, 2000)
    M = len(idx)
    hid = gen_device.hidden(wl, dev)
    x_bits = host_bits(hid)
    ctx = _ctx(model, wl.N, M)
    didx = dev_i32(idx)
    h_dev, g_dev = hid, didx                 # the device's own chain
    h_ref, g_ref = x_bits, idx               # the oracle's own chain
    lines = []
    for l in range(n_layers):
        wd = gen_device.layer_weights(model, l, wl.seed, dev)
        Kd0, Vd0 = gen_device.cache(wl, l, dev)
        w = {k: (None if v is None else host_bits(v)) for k, v in wd.items()}
        Ks, Vs = host_bits(Kd0), host_bits(Vd0)
        ref = layer.recompute_layer(h_ref, g_ref, Ks, Vs, idx, w, model)           # all M rows: the next layer needs them
        dw = cc.LayerWeights(**wd)
        # (a) teacher-forced: the device gets the oracle's input of this layer
        Kd, Vd = Kd0.clone(), Vd0.clone()
        out_tf = torch.empty((M, model.d), dtype=torch.bfloat16, device=dev)
        h_tf = hid if l == 0 else dev_bf16(h_ref)
        ctx.recompute_layer(h_tf, didx if l == 0 else None, cc.KVLayer(Kd, Vd), didx, M, dw, out_tf,
                            _lib.FLAG_CHECK_IDX)
        torch.cuda.synchronize()
        got = dict(out=host_bits(out_tf), K=host_bits(Kd), V=host_bits(Vd))
        _assert_layer(got, ref, Ks, Vs, idx, f"stack layer {l} teacher-forced")
        tf_mx, tf_mn = err_stats(bits_f64(got["out"]), ref.out)
        # (b) chained: the device continues from its own output
        Kc, Vc = Kd0, Vd0
        out_ch = torch.empty((M, model.d), dtype=torch.bfloat16, device=dev)
        ctx.recompute_layer(h_dev, g_dev, cc.KVLayer(Kc, Vc), didx, M, dw, out_ch, 0)
        torch.cuda.synchronize()
        ch_mx, ch_mn = err_stats(bits_f64(host_bits(out_ch)), ref.out)
        kv_mx, _ = err_stats(bits_f64(host_bits(Kc)[idx]), ref.k_new)
        lines.append(f"layer {l}: teacher-forced out max {tf_mx:.2e} mean {tf_mn:.2e} | chained out max {ch_mx:.2e} "
                     f"mean {ch_mn:.2e}, K max {kv_mx:.2e} | rms(out) {np.sqrt(np.mean(ref.out ** 2)):.2f}")
        assert np.isfinite(bits_f64(host_bits(out_ch))).all()
        assert ch_mn <= 10 * MEAN_ABS and ch_mx <= 0.5, (l, ch_mx, ch_mn)          # no blow-up with depth
        h_dev, g_dev = out_ch, None
        h_ref, g_ref = ref.out_bits, None
        del wd, dw, Kd, Vd, Kd0, Vd0
    ctx.close()
    with capsys.disabled():
        print(f"\nstack drift, 8 layers of the 4k shape at 20 percent (M = {M}):\n  " + "\n  ".join(lines))


@pytest.mark.parametrize("prefix", [16, 0])
def test_whole_request_on_the_device(prefix):
    """A request from the offline artefacts to the last layer's output, every step on the
    device: scores from the batched auxiliary attention tensors -> candidates -> grouping,
    per-chunk caches assembled behind one prefix copy (or none), two layers recomputed on the
    selected rows.  The oracle does the same from the same inputs."""
    from oracle import select as osel
    wl = replace(CONFIGS["C1x2"], P=prefix, chunk_lens=(256, 200, 300, 129))
    model = wl.model
    ws = [gen.layer_weights(model, l, wl.seed) for l in range(2)]
    xl, _ = gen.hidden_pair(wl)
    per = fixture.chunk_caches(xl, wl.P, wl.chunk_lens, ws, model)
    blocks = gen.aux_attention_blocks(wl, heads=4)
    # oracle
    idx = osel.select_from_scores(osel.block_scores(blocks), 2000, wl.window, wl.tau, True, wl.P, wl.Q)
    Ks, Vs = fixture.concat_caches(per, wl.P, wl.chunk_lens, wl.Q, model, 2)
    ref = fixture.selective_prefill(xl, Ks, Vs, idx, ws, model)
    # device
    ctx = _ctx(model, wl.N, wl.N)
    dblocks = [(torch.from_numpy(A).to(DEV), c0, L) for A, c0, L in blocks]
    didx, M = ctx.select_blocks(dblocks, 2000, wl.window, wl.tau, 0, wl.P, wl.Q)
    assert M == len(idx) and np.array_equal(didx[:M].cpu().numpy(), idx)
    h, g = dev_bf16(xl), didx
    for l in range(2):
        Kd = torch.empty((wl.N, model.H_kv, model.d_h), dtype=torch.bfloat16, device=DEV)
        Vd = torch.empty_like(Kd)
        ctx.assemble_cache([dev_bf16(pc[0][l]) for pc in per], [dev_bf16(pc[1][l]) for pc in per],
                           wl.P, wl.Q, cc.KVLayer(Kd, Vd))
        torch.cuda.synchronize()
        assert np.array_equal(host_bits(Vd), Vs[l])
        assert (host_bits(Kd) == Ks[l]).mean() > 0.995          # re-rotated keys: same value up to one rounding
        out = torch.empty((M, model.d), dtype=torch.bfloat16, device=DEV)
        ctx.recompute_layer(h, g, cc.KVLayer(Kd, Vd), didx, M, dev_weights(ws[l]), out, _lib.FLAG_CHECK_IDX)
        torch.cuda.synchronize()
        mx, mn = err_stats(bits_f64(host_bits(out)), ref[l].out)
        print(f"request P={prefix} layer {l}: M={M} out max {mx:.2e} mean {mn:.2e}")
        # chained on the device's own outputs and keys: one bf16 spacing of the residual
        # stream on top of the per-layer bound (as in the stack test above)
        assert mx <= MAX_ABS + 2.0 ** -7 * np.abs(ref[l].out).max() and mn <= MEAN_ABS
        for name, fresh, got in (("K", ref[l].k_new, Kd), ("V", ref[l].v_new, Vd)):
            kmx, kmn = err_stats(bits_f64(host_bits(got)[idx]), fresh)
            assert kmx <= MAX_ABS + (2.0 ** -7 * np.abs(fresh).max() if l else 0.0) and kmn <= MEAN_ABS, (name, l, kmx, kmn)
        h, g = out, None
    ctx.close()


def _stratified_rows(M, g, n_extra, seed):
    """The rows whose layer output is compared in a full-size case: the first and the last, one
    (drawn at random) in every block of 256 (token, head) columns that an attention workgroup
    owns, one in every aligned group of 128 rows where those blocks are wider than that (every
    128-, 192- and 256-row GEMM tile then holds a sampled row), and n_extra more at random."""
    rng = np.random.default_rng(seed)
    cols = M * g
    picks = [0, M - 1]
    for b in range((cols + 255) // 256):
        picks.append(int(rng.integers(256 * b, min(cols, 256 * b + 256))) // g)
    if 256 // g > 64:
        for r0 in range(0, M, 128):
            picks.append(int(rng.integers(r0, min(M, r0 + 128))))
    picks += [int(v) for v in rng.choice(M, size=min(n_extra, M), replace=False)]
    return np.unique(np.asarray(picks, dtype=np.int64))


def _sampled_layer_case(name, bp, n_extra, seed):
    wl = CONFIGS[name]
    model = replace(wl.model, n_layers=1)
    w = gen.layer_weights(model, 0, wl.seed)
    xl, xg = gen.hidden_pair(wl)
    Ks, Vs = fixture.stale_cache_one_layer(xl, w, model)
    Ks[wl.P + wl.T:], Vs[wl.P + wl.T:] = 0, 0
    idx = gen.exact_ratio_idx(wl, bp)
    M = len(idx)
    rows = _stratified_rows(M, model.g, n_extra, seed)
    got, ref = _run_layer(model, xg, idx, Ks, Vs, idx, w, rows=rows)
    _assert_layer(got, ref, Ks, Vs, idx, f"{name}@{bp // 100}% M={M} ({len(rows)} rows compared)")


@pytest.mark.parametrize("bp", [1000, 2000, 4000])
def test_llama8b_layer_4k_sampled_rows(bp):
    _sampled_layer_case("C2", bp, 16, bp)


def test_llama8b_layer_16k_bench_shape_sampled_rows():
    """The shape and launch configuration bench.py times (one layer of it)."""
    _sampled_layer_case("C3", 2000, 16, 7)


def _device_drawn_layer_case(name, bp, n_extra, seed, dense=False):
    """One layer at a config's full size with inputs drawn on the device (torch's
    generator; the host streams would take minutes at these sizes) and copied to the
    host for the oracle, which projects keys and values for every recomputed row and
    evaluates attention and the rest of the layer for a stratified sample of rows.
    dense: every cache slot is recomputed (idx = 0..N-1), the full-prefill launch."""
    from workloads import gen_device
    wl = CONFIGS[name]
    model = replace(wl.model, n_layers=1)
    dev = torch.device(DEV)
    wd = gen_device.layer_weights(model, 0, wl.seed, dev)
    hid = gen_device.hidden(wl, dev)
    Kd, Vd = gen_device.cache(wl, 0, dev)
    w = {k: (None if v is None else host_bits(v)) for k, v in wd.items()}
    xg, Ks, Vs = host_bits(hid), host_bits(Kd), host_bits(Vd)
    idx = np.arange(wl.N, dtype=np.int32) if dense else gen.exact_ratio_idx(wl, bp)
    M = len(idx)
    rows = _stratified_rows(M, model.g, n_extra, seed)
    ctx = _ctx(model, wl.N, M)
    out = torch.full((M, model.d), float("nan"), dtype=torch.bfloat16, device=dev)
    didx = dev_i32(idx)
    ctx.recompute_layer(hid, didx, cc.KVLayer(Kd, Vd), didx, M, cc.LayerWeights(**wd), out,
                        _lib.FLAG_CHECK_IDX)
    torch.cuda.synchronize()
    got = dict(out=host_bits(out), K=host_bits(Kd), V=host_bits(Vd))
    ctx.close()
    del wd, hid, Kd, Vd, out
    torch.cuda.empty_cache()
    ref = layer.recompute_layer(xg, idx, Ks, Vs, idx, w, model, rows=rows, q_for_rows_only=True)
    tag = f"{name} dense" if dense else f"{name}@{bp // 100}%"
    _assert_layer(got, ref, Ks, Vs, idx, f"{tag} M={M} ({len(rows)} rows compared)")


@pytest.mark.parametrize("bp", [500, 2000, 5000])
def test_qwen7b_layer_29k_ragged_chunks_sampled_rows(bp):
    """C4: 28 q / 4 kv heads (groups of 7), QKV bias, chunk lengths U[256,1536]; 5 % (split
    attention, split-K projections), 20 % and 50 % (the most rows of any config)."""
    _device_drawn_layer_case("C4", bp, 16, 11 + bp)


def test_llama70b_layer_64k_sampled_rows():
    """C5: d = 8192, 64 q / 8 kv heads, 64k context."""
    _device_drawn_layer_case("C5", 2000, 32, 12)


def test_llama8b_layer_16k_every_slot_recomputed():
    """Full prefill on the same kernels, at the size bench.py times it (Section 5.1 "Full
    Attention", the reference point of the efficiency table of Section 5.6): every one of the
    16576 cache slots of the 16k workload is recomputed in one call (idx = 0..N-1).  Every K/V row
    against the oracle, the layer output on the stratified sample."""
    _device_drawn_layer_case("C3", 0, 16, 13, dense=True)
