"""Seeded generators: hidden rows, layer weights, auxiliary attention blocks.

Counter-based Philox streams keyed by (seed, stream id) so that every array
can be regenerated on its own.  bf16 arrays are returned as uint16 bit
patterns (numpy has no bf16 dtype); ``bf16_to_f32`` widens them exactly.
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np

from .configs import ModelShape, Workload

# stream ids
_S_HIDDEN, _S_DELTA, _S_SCORES, _S_WEIGHTS, _S_IDX = 1, 2, 3, 100, 7


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_bf16(rng: np.random.Generator, shape, std: float, mean: float = 0.0) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    if mean != 0.0:
        x += np.float32(mean)
    return f32_to_bf16_bits(x)


def hidden_pair(wl: Workload, delta_std: float = 0.5) -> Tuple[np.ndarray, np.ndarray]:
    """(X_local, X_glob), both bf16 bits [N, d].

    X_local stands for the hidden rows each chunk saw when it was prefilled on
    its own; X_glob for the rows the same tokens have when the whole context is
    visible.  They differ on chunk tokens only (prefix rows see the same context
    either way; query rows have no precomputed state at all).
    """
    m = wl.model
    x = _rng(wl.seed, _S_HIDDEN).standard_normal(size=(wl.N, m.d), dtype=np.float32)
    xl = f32_to_bf16_bits(x)
    dl = _rng(wl.seed, _S_DELTA).standard_normal(size=(wl.T, m.d), dtype=np.float32)
    dl *= np.float32(delta_std)
    xg = x.copy()
    xg[wl.P:wl.P + wl.T] += dl
    return xl, f32_to_bf16_bits(xg)


def layer_weights(model: ModelShape, layer: int, seed: int) -> Dict[str, np.ndarray]:
    """bf16 bits of one decoder layer.  Matrices are [out_features, in_features]
    row-major (y = W x).  ``w_qkv`` stacks the q, k and v projections by rows."""
    r = _rng(seed, _S_WEIGHTS + layer)
    d, f, nq = model.d, model.f, model.n_qkv
    si, so = model.sigma_in, model.sigma_out
    w = {
        "w_in_norm": _normal_bf16(r, (d,), 0.1, 1.0),
        "w_qkv": _normal_bf16(r, (nq, d), si),
        "b_qkv": _normal_bf16(r, (nq,), 0.1) if model.qkv_bias else None,
        "w_o": _normal_bf16(r, (d, model.H_q * model.d_h), so),
        "w_post_norm": _normal_bf16(r, (d,), 0.1, 1.0),
        "w_gate": _normal_bf16(r, (f, d), si),
        "w_up": _normal_bf16(r, (f, d), si),
        "w_down": _normal_bf16(r, (d, f), so),
    }
    return w


def _row_softmax(z: np.ndarray) -> np.ndarray:
    z = z - z.max(axis=1, keepdims=True)
    e = np.exp(z)
    return (e / e.sum(axis=1, keepdims=True)).astype(np.float32)


def aux_attention(wl: Workload) -> np.ndarray:
    """fp32 [Q_a, T]: the query->chunk block of an auxiliary model's last-layer
    attention, synthesised.  Rows are softmaxes over the T chunk tokens.

    spikes   : N(0,1) logits plus 8 spikes of +6 at random columns per row.
    heavy    : 2*N(0,1) logits plus T/64 bumps of +4 shared by all rows over
               spans of U[4,24] tokens (about a fifth of the tokens), so that high
               column sums come in runs and a recompute ratio of 20 % ends up
               with roughly 20 % of the tokens after grouping (a few tokens
               carry most of the mass, as the paper observes).
    boundary : heavy, with the bump starts drawn within +-32 tokens of chunk
               starts (attention-sink-like mass at chunk boundaries).
    """
    r = _rng(wl.seed, _S_SCORES)
    Qa, T = wl.Q_a, wl.T
    z = r.standard_normal(size=(Qa, T), dtype=np.float32).astype(np.float64)
    if wl.score_kind == "spikes":
        for q in range(Qa):
            cols = r.choice(T, size=8, replace=False)
            z[q, cols] += 6.0
    else:
        z *= 2.0
        n_bumps = max(1, T // 64)
        lens = r.integers(4, 25, size=n_bumps)
        if wl.score_kind == "boundary":
            starts_c = np.asarray(wl.chunk_starts)
            base = starts_c[r.integers(0, len(starts_c), size=n_bumps)]
            starts = np.clip(base + r.integers(-32, 33, size=n_bumps), 0, T - 1)
        else:
            starts = r.integers(0, T, size=n_bumps)
        for s, L in zip(starts, lens):
            z[:, int(s):min(T, int(s + L))] += 4.0
    return _row_softmax(z)


def aux_attention_blocks(wl: Workload, heads: int, prefix: int | None = None):
    """The batched form of the auxiliary model's last-layer attention (one element per
    `chunk c + query`): list of (A fp32 [heads, Q_a, P + L_c + Q_a], col0 = P, L_c).
    Every row is a softmax over that element's own key columns (prefix, chunk, the query's
    causal part), so the scores are normalised per chunk.  Logits: 2*N(0,1) per head, plus
    bumps of +4 over spans of U[4,24] chunk tokens shared by all heads and rows (about L_c/64
    per chunk), plus +2 on the first prefix column (a sink) when there is a prefix."""
    P = wl.P if prefix is None else prefix
    r = _rng(wl.seed, _S_SCORES + 17)
    Qa = wl.Q_a
    out = []
    for L in wl.chunk_lens:
        W = P + L + Qa
        z = 2.0 * r.standard_normal(size=(heads, Qa, W), dtype=np.float32).astype(np.float64)
        for _ in range(max(1, L // 64)):
            s0 = int(r.integers(0, L))
            z[:, :, P + s0:P + min(L, s0 + int(r.integers(4, 25)))] += 4.0
        if P > 0:
            z[:, :, 0] += 2.0
        q = np.arange(Qa)[:, None]
        k = np.arange(W)[None, :]
        z = np.where(k <= P + L + q, z, -np.inf)       # the query rows are causal among themselves
        z -= z.max(axis=-1, keepdims=True)
        e = np.exp(z)
        out.append(((e / e.sum(axis=-1, keepdims=True)).astype(np.float32), P, int(L)))
    return out


def exact_ratio_idx(wl: Workload, recomp_bp: int, run: int | None = None) -> np.ndarray:
    """A hand-built recompute set of exactly floor(T*bp/10000) chunk tokens made
    of non-overlapping runs of ``run`` tokens at random starts (what grouping
    produces, but with a size that does not depend on the scores), followed by
    the Q query slots.  int32, strictly ascending, cache-slot numbering."""
    run = wl.window if run is None else run
    T = wl.T
    k = T * recomp_bp // 10000
    r = _rng(wl.seed, _S_IDX + recomp_bp)
    n_runs, rem = divmod(k, run)
    n_slots = T // run
    slots = np.sort(r.choice(n_slots, size=min(n_slots, n_runs + (1 if rem else 0)), replace=False))
    marks = np.zeros(T, dtype=bool)
    for j, s in enumerate(slots):
        L = run if j < n_runs else rem
        marks[s * run:s * run + L] = True
    sel = np.nonzero(marks)[0][:k]
    tail = np.arange(wl.P + T, wl.N)
    return np.concatenate([sel + wl.P, tail]).astype(np.int32)


def random_cache(wl: Workload, std: float = 0.6) -> Tuple[np.ndarray, np.ndarray]:
    """bf16 bits of a K and a V cache [N, H_kv, d_h] filled with N(0, std):
    stands in for a stale cache when only speed is measured."""
    m = wl.model
    r = _rng(wl.seed, 55)
    return (_normal_bf16(r, (wl.N, m.H_kv, m.d_h), std),
            _normal_bf16(r, (wl.N, m.H_kv, m.d_h), std))
