"""Oracle for the selective recompute of one decoder layer (Section 4.3, "KV
cache update": the primary model recomputes the selected tokens with position
ids consistent with full attention and overwrites their entries in the global
KV cache).  The layer is the pre-norm GQA decoder layer of the paper's primary
models (Section 5.1 names Qwen2.5 / LLaMA-3 style models): RMSNorm, QKV
projection, rotary embedding, causal softmax attention, output projection,
residual, RMSNorm, SwiGLU MLP, residual.

Test infrastructure: never imported by the product path.  fp64 throughout;
the only rounding is where the data structure itself is bf16: the K/V rows
written into the cache.  Attention reads the cache as stored (rounded).

Readings where the paper is silent: rotary pairs are (j, j + d_h/2) with
angle pos * base**(-2j/d_h), no frequency scaling; the position of cache slot
j is j; every selected row's K/V is written before any attention row is
evaluated; hidden rows above the first layer are the compact output of the
layer below.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional, Sequence

import numpy as np

from . import bf16


@dataclass
class LayerResult:
    out: np.ndarray            # fp64 [R, d] layer output rows (R = len(rows))
    out_bits: np.ndarray       # the same rounded to bf16 (uint16)
    rows: np.ndarray           # which of the M recomputed rows were evaluated
    k_new: np.ndarray          # fp64 [M, H_kv, d_h] rotated keys before rounding
    v_new: np.ndarray          # fp64 [M, H_kv, d_h] values before rounding
    K_bits: np.ndarray         # updated cache, uint16 [N, H_kv, d_h]
    V_bits: np.ndarray
    attn_out: np.ndarray       # fp64 [R, H_q*d_h] attention output (before W_o)
    q_rot: np.ndarray          # fp64 [M, H_q, d_h] rotated queries
    row_sums: np.ndarray       # fp64 [R, H_q] sum of attention probabilities
    y: np.ndarray              # fp64 [R, d] residual stream after attention


def _w(weights: Dict[str, np.ndarray], name: str) -> Optional[np.ndarray]:
    b = weights.get(name)
    return None if b is None else bf16.bits_to_f64(b)


def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    """x * rsqrt(mean(x^2) + eps) * w, per row."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * w


def rope_rotate(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotary embedding of x [M, H, d_h] at integer positions pos [M].
    Component j (< d_h/2) pairs with j + d_h/2; the pair is turned by the
    angle pos * base**(-2j/d_h)."""
    d_h = x.shape[-1]
    half = d_h // 2
    inv = base ** (-2.0 * np.arange(half, dtype=np.float64) / d_h)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv[None, :]      # [M, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def qkv_rows(x: np.ndarray, weights, model, pos: np.ndarray):
    """Steps 1-3 for rows x [M, d] at positions pos: normalise, project, rotate.
    Returns (q [M,H_q,d_h], k [M,H_kv,d_h], v [M,H_kv,d_h]) in fp64."""
    M = x.shape[0]
    n = rmsnorm(x, _w(weights, "w_in_norm"), model.rms_eps)
    qkv = n @ _w(weights, "w_qkv").T
    b = _w(weights, "b_qkv")
    if b is not None:
        qkv = qkv + b
    nq, nk = model.H_q * model.d_h, model.H_kv * model.d_h
    q = qkv[:, :nq].reshape(M, model.H_q, model.d_h)
    k = qkv[:, nq:nq + nk].reshape(M, model.H_kv, model.d_h)
    v = qkv[:, nq + nk:].reshape(M, model.H_kv, model.d_h)
    return rope_rotate(q, pos, model.rope_base), rope_rotate(k, pos, model.rope_base), v


def kv_rows(x: np.ndarray, weights, model, pos: np.ndarray):
    """Steps 1-3 restricted to the key and value heads (the rows of W_qkv below the
    query heads): (k [M,H_kv,d_h] rotated, v [M,H_kv,d_h]) in fp64.  Same numbers as
    the k and v of qkv_rows; used where the queries of most rows are not needed."""
    M = x.shape[0]
    nq, nk = model.H_q * model.d_h, model.H_kv * model.d_h
    n = rmsnorm(x, _w(weights, "w_in_norm"), model.rms_eps)
    kv = n @ bf16.bits_to_f64(weights["w_qkv"][nq:]).T
    if weights.get("b_qkv") is not None:
        kv = kv + bf16.bits_to_f64(weights["b_qkv"][nq:])
    k = kv[:, :nk].reshape(M, model.H_kv, model.d_h)
    v = kv[:, nk:].reshape(M, model.H_kv, model.d_h)
    return rope_rotate(k, pos, model.rope_base), v


def attend_row(q_row: np.ndarray, K: np.ndarray, V: np.ndarray, p: int, g: int):
    """Causal GQA attention of one query row (all heads) at position p over
    cache slots 0..p.  q_row [H_q, d_h]; K, V fp64 [N, H_kv, d_h].
    Returns (o [H_q, d_h], probs [H_q, p+1])."""
    H_q, d_h = q_row.shape
    H_kv = H_q // g
    qg = q_row.reshape(H_kv, g, d_h)
    # per kv head k: logits[k] = qg[k] K[:p+1, k, :]^T and o[k] = probs[k] V[:p+1, k, :], as
    # two batched library matrix products (batch index = kv head)
    logits = np.matmul(qg, K[:p + 1].transpose(1, 2, 0)) / np.sqrt(float(d_h))      # [H_kv, g, p+1]
    logits = logits - logits.max(axis=-1, keepdims=True)
    e = np.exp(logits)
    probs = e / e.sum(axis=-1, keepdims=True)
    o = np.matmul(probs, V[:p + 1].transpose(1, 0, 2))                               # [H_kv, g, d_h]
    return o.reshape(H_q, d_h), probs.reshape(H_q, p + 1)


def recompute_layer(hidden_bits: np.ndarray, gather_idx: Optional[np.ndarray],
                    K_bits: np.ndarray, V_bits: np.ndarray, idx: np.ndarray,
                    weights: Dict[str, np.ndarray], model,
                    rows: Optional[Sequence[int]] = None,
                    q_for_rows_only: bool = False) -> LayerResult:
    """Selective recompute of one layer.

    hidden_bits : bf16 bits [rows_in, d]; row gather_idx[i] (or row i when
                  gather_idx is None) is the layer input of recomputed token i.
    K_bits/V_bits : bf16 bits [N, H_kv, d_h], the global cache of this layer
                  (not modified; the updated copy is returned).
    idx         : int [M] strictly ascending cache slots = global positions.
    rows        : evaluate attention and the rest of the layer only for these
                  of the M rows (they are independent once the cache is
                  updated); None = all.
    q_for_rows_only : project queries only for `rows` (keys and values are still
                  computed for all M rows); q_rot then holds zeros elsewhere.
    """
    idx = np.asarray(idx, dtype=np.int64)
    M = idx.shape[0]
    g = model.g
    src = np.arange(M) if gather_idx is None else np.asarray(gather_idx, dtype=np.int64)
    x = bf16.bits_to_f64(hidden_bits[src])                              # step 1: gather
    if q_for_rows_only and rows is not None:
        k, v = kv_rows(x, weights, model, idx)                          # steps 1-3, k and v
        rsel = np.asarray(rows, dtype=np.int64)
        q = np.zeros((M, model.H_q, model.d_h))
        q[rsel] = qkv_rows(x[rsel], weights, model, idx[rsel])[0]       # steps 1-3, q of the sample
    else:
        q, k, v = qkv_rows(x, weights, model, idx)                      # steps 1-3
    K_new, V_new = K_bits.copy(), V_bits.copy()
    K_new[idx] = bf16.f64_to_bits(k)                                    # step 4: overwrite
    V_new[idx] = bf16.f64_to_bits(v)
    Kf, Vf = bf16.bits_to_f64(K_new), bf16.bits_to_f64(V_new)

    rows = np.arange(M) if rows is None else np.asarray(rows, dtype=np.int64)
    R = rows.shape[0]
    attn = np.zeros((R, model.H_q * model.d_h))
    sums = np.zeros((R, model.H_q))
    for r, i in enumerate(rows):                                        # step 5
        o, probs = attend_row(q[i], Kf, Vf, int(idx[i]), g)
        attn[r] = o.reshape(-1)
        sums[r] = probs.sum(axis=-1)
    y = x[rows] + attn @ _w(weights, "w_o").T                           # step 6
    m = rmsnorm(y, _w(weights, "w_post_norm"), model.rms_eps)           # step 7
    act = silu(m @ _w(weights, "w_gate").T) * (m @ _w(weights, "w_up").T)
    z = y + act @ _w(weights, "w_down").T
    return LayerResult(out=z, out_bits=bf16.f64_to_bits(z), rows=rows, k_new=k, v_new=v,
                       K_bits=K_new, V_bits=V_new, attn_out=attn, q_rot=q,
                       row_sums=sums, y=y)
