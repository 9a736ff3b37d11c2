"""Oracle-side fixtures: dense causal prefill, the offline per-chunk prefill
behind a shared prefix, and the online concatenation with re-numbered
positions (Section 4.1), plus the layer-by-layer drivers.

Test infrastructure: never imported by the product path.  These build the
stale caches that the selective recompute starts from and the full-attention
result it must reproduce when every token is recomputed.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import bf16
from .layer import LayerResult, _w, qkv_rows, recompute_layer, rmsnorm, rope_rotate, silu


def dense_layer(x: np.ndarray, pos: np.ndarray, weights, model
                ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """One decoder layer over a whole token sequence x [n, d] (fp64) with
    causal attention in array order and rotary positions ``pos``.  This is
    ordinary full-attention prefill ("Full Attention" in Section 5.1), written
    in matrix form.  K/V are rounded to bf16 as a cache stores them and
    attention reads the rounded values.  Returns (out fp64 [n,d], K bits, V bits)."""
    n = x.shape[0]
    q, k, v = qkv_rows(x, weights, model, pos)
    Kb, Vb = bf16.f64_to_bits(k), bf16.f64_to_bits(v)
    Kf, Vf = bf16.bits_to_f64(Kb), bf16.bits_to_f64(Vb)
    g = model.g
    Kh = np.repeat(Kf, g, axis=1)                      # [n, H_q, d_h]
    Vh = np.repeat(Vf, g, axis=1)
    logits = np.einsum("ihd,jhd->hij", q, Kh) / np.sqrt(float(model.d_h))
    mask = np.tril(np.ones((n, n), dtype=bool))
    logits = np.where(mask[None], logits, -np.inf)
    logits = logits - logits.max(axis=-1, keepdims=True)
    e = np.exp(logits)
    p = e / e.sum(axis=-1, keepdims=True)
    o = np.einsum("hij,jhd->ihd", p, Vh).reshape(n, -1)
    y = x + o @ _w(weights, "w_o").T
    m = rmsnorm(y, _w(weights, "w_post_norm"), model.rms_eps)
    z = y + (silu(m @ _w(weights, "w_gate").T) * (m @ _w(weights, "w_up").T)) @ _w(weights, "w_down").T
    return z, Kb, Vb


def full_prefill(x_bits: np.ndarray, weights_list: Sequence[Dict], model):
    """Dense prefill of a stack over all N tokens at positions 0..N-1.
    Layer outputs are rounded to bf16 between layers.  Returns
    (final hidden bits [N,d], [K bits per layer], [V bits per layer])."""
    n = x_bits.shape[0]
    pos = np.arange(n)
    h = x_bits
    Ks, Vs = [], []
    for w in weights_list:
        z, Kb, Vb = dense_layer(bf16.bits_to_f64(h), pos, w, model)
        Ks.append(Kb)
        Vs.append(Vb)
        h = bf16.f64_to_bits(z)
    return h, Ks, Vs


def rerotate_keys(K_bits: np.ndarray, delta: int, model) -> np.ndarray:
    """Move stored keys from position p to p + delta: rotary rotations add, so
    this is one more rotation by ``delta`` (position-id rearrangement,
    Section 4.1), applied to the bf16 cache rows and rounded again."""
    n = K_bits.shape[0]
    k = rope_rotate(bf16.bits_to_f64(K_bits), np.full(n, delta), model.rope_base)
    return bf16.f64_to_bits(k)


def chunk_caches(x_bits: np.ndarray, P: int, chunk_lens: Sequence[int],
                 weights_list: Sequence[Dict], model):
    """Offline phase (Section 4.1): every chunk is prefilled alone behind the
    shared prefix, at local positions 0..P+L_c-1.  x_bits [N, d] holds the
    prefix rows, then the chunk rows in order (query rows are ignored).
    Returns, per chunk, ([K bits per layer], [V bits per layer]) of shape
    [P+L_c, H_kv, d_h]."""
    out = []
    s = P
    for L in chunk_lens:
        rows = np.concatenate([np.arange(P), np.arange(s, s + L)])
        _, Ks, Vs = full_prefill(x_bits[rows], weights_list, model)
        out.append((Ks, Vs))
        s += L
    return out


def concat_caches(per_chunk, P: int, chunk_lens: Sequence[int], Q: int, model, n_layers: int):
    """Online assembly (Section 4.1): keep the prefix rows of the first chunk
    only, append every chunk's own rows, and give chunk c the position range
    that follows chunk c-1 by re-rotating its keys.  The Q query slots at the
    end hold zeros (nothing was precomputed for them).
    Returns ([K bits per layer], [V bits per layer]) of shape [N, H_kv, d_h]."""
    Kg, Vg = [], []
    for l in range(n_layers):
        Kparts = [per_chunk[0][0][l][:P]]
        Vparts = [per_chunk[0][1][l][:P]]
        start = 0
        for c, L in enumerate(chunk_lens):
            Kc, Vc = per_chunk[c][0][l][P:], per_chunk[c][1][l][P:]
            Kparts.append(rerotate_keys(Kc, start, model) if start else Kc)
            Vparts.append(Vc)
            start += L
        tail = np.zeros((Q,) + Kparts[0].shape[1:], dtype=np.uint16)
        Kg.append(np.concatenate(Kparts + [tail]))
        Vg.append(np.concatenate(Vparts + [tail]))
    return Kg, Vg


def stale_caches(x_bits, P, chunk_lens, Q, weights_list, model):
    per_chunk = chunk_caches(x_bits, P, chunk_lens, weights_list, model)
    return concat_caches(per_chunk, P, chunk_lens, Q, model, len(weights_list))


def stale_cache_one_layer(x_local_bits, weights, model):
    """Single-layer shortcut: pre-rotation K/V of a token depend on its own
    hidden row only, and re-rotation composes, so the concatenated cache of a
    layer whose inputs were ``x_local`` equals that layer's K/V at global
    positions.  (Differs from the two-step build only by one bf16 rounding of
    the re-rotated keys.)"""
    n = x_local_bits.shape[0]
    _, k, v = qkv_rows(bf16.bits_to_f64(x_local_bits), weights, model, np.arange(n))
    return bf16.f64_to_bits(k), bf16.f64_to_bits(v)


def selective_prefill(x_bits: np.ndarray, Ks: List[np.ndarray], Vs: List[np.ndarray],
                      idx: np.ndarray, weights_list: Sequence[Dict], model,
                      rows_last: Optional[Sequence[int]] = None) -> List[LayerResult]:
    """Layer-by-layer selective recompute of a stack.  Layer 0 gathers rows
    ``idx`` of x_bits [N, d]; every later layer takes the compact bf16 output
    of the layer below.  Returns the per-layer results."""
    results = []
    h, gidx = x_bits, np.asarray(idx)
    for l, w in enumerate(weights_list):
        last = l == len(weights_list) - 1
        r = recompute_layer(h, gidx, Ks[l], Vs[l], idx, w, model,
                            rows=rows_last if last else None)
        results.append(r)
        h, gidx = r.out_bits, None
    return results
