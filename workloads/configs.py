"""Shapes of the synthetic RAG workloads (model shape + sequence layout).

The paper evaluates with ~1000-token chunks behind a shared system-prompt
prefix, a short user query at the end, and 4K-16K contexts (Section 5.1,
Section 5.6); its primary models are 8B-14B GQA decoders.  The workloads
below take those shapes at five sizes.  Nothing here is the method itself.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Tuple

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    d: int            # hidden width
    H_q: int          # query heads
    H_kv: int         # key/value heads
    d_h: int          # head dim
    f: int            # SwiGLU inner width
    rope_base: float
    rms_eps: float
    qkv_bias: bool
    n_layers: int

    @property
    def g(self) -> int:
        return self.H_q // self.H_kv

    @property
    def n_qkv(self) -> int:
        return (self.H_q + 2 * self.H_kv) * self.d_h

    @property
    def sigma_in(self) -> float:
        """std of the input-side matrices (Wqkv, Wgate, Wup): 0.02 capped by
        the fan-in-scaled "small init" sqrt(2/(5 d)) so that pre-activations
        stay O(1) at every width."""
        return min(0.02, math.sqrt(2.0 / (5.0 * self.d)))

    @property
    def sigma_out(self) -> float:
        """std of the output-side matrices (Wo, Wdown): input-side std divided
        by sqrt(depth) so that the residual stream of a stack stays O(1)."""
        return self.sigma_in / math.sqrt(self.n_layers)


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelShape
    P: int                        # shared-prefix tokens
    chunk_lens: Tuple[int, ...]   # L_c per chunk
    Q: int                        # user-query tokens (tail of the cache)
    Q_a: int                      # rows of the auxiliary attention block
    recomp_bp: Tuple[int, ...]    # recompute ratios, basis points
    window: int
    tau: int
    seed: int
    score_kind: str               # "spikes" | "heavy" | "boundary"

    @property
    def T(self) -> int:
        return int(sum(self.chunk_lens))

    @property
    def N(self) -> int:
        return self.P + self.T + self.Q

    @property
    def chunk_starts(self) -> Tuple[int, ...]:
        """Start of each chunk on the chunk-token axis (0-based, prefix excluded)."""
        out, s = [], 0
        for L in self.chunk_lens:
            out.append(s)
            s += L
        return tuple(out)


_TINY = ModelShape(d=256, H_q=4, H_kv=2, d_h=64, f=1024, rope_base=1.0e4,
                   rms_eps=1e-5, qkv_bias=False, n_layers=1)
_L8B = ModelShape(d=4096, H_q=32, H_kv=8, d_h=128, f=14336, rope_base=5.0e5,
                  rms_eps=1e-5, qkv_bias=False, n_layers=1)
_Q7B = ModelShape(d=3584, H_q=28, H_kv=4, d_h=128, f=18944, rope_base=1.0e6,
                  rms_eps=1e-6, qkv_bias=True, n_layers=28)
_L70B = ModelShape(d=8192, H_q=64, H_kv=8, d_h=128, f=28672, rope_base=5.0e5,
                   rms_eps=1e-5, qkv_bias=False, n_layers=1)


def _c4_chunks(seed: int = 3) -> Tuple[int, ...]:
    rng = np.random.Generator(np.random.Philox(key=[seed, 0xC4]))
    return tuple(int(v) for v in rng.integers(256, 1537, size=32))


CONFIGS = {
    # configs[0]
    "C1": Workload("C1", _TINY, P=16, chunk_lens=(256,) * 4, Q=32, Q_a=32,
                   recomp_bp=(2000,), window=8, tau=5, seed=0, score_kind="spikes"),
    # configs[1]
    "C2": Workload("C2", _L8B, P=64, chunk_lens=(512,) * 8, Q=64, Q_a=64,
                   recomp_bp=(1000, 2000, 4000), window=16, tau=10, seed=1,
                   score_kind="heavy"),
    # configs[2]: the 32-layer stack at 16k context
    "C3": Workload("C3", replace(_L8B, n_layers=32), P=64, chunk_lens=(1024,) * 16,
                   Q=128, Q_a=128, recomp_bp=(2000,), window=16, tau=10, seed=2,
                   score_kind="heavy"),
    # configs[3]
    "C4": Workload("C4", _Q7B, P=64, chunk_lens=_c4_chunks(), Q=128, Q_a=128,
                   recomp_bp=(500, 2000, 5000), window=16, tau=10, seed=3,
                   score_kind="boundary"),
    # configs[4]
    "C5": Workload("C5", _L70B, P=64, chunk_lens=(1024,) * 64, Q=256, Q_a=256,
                   recomp_bp=(2000,), window=32, tau=20, seed=4, score_kind="heavy"),
    # two-layer variant of C1 so that stale caches differ from fresh ones
    "C1x2": Workload("C1x2", replace(_TINY, n_layers=2), P=16, chunk_lens=(256,) * 4,
                     Q=32, Q_a=32, recomp_bp=(2000,), window=8, tau=5, seed=5,
                     score_kind="spikes"),
}


def get_workload(name: str) -> Workload:
    return CONFIGS[name]
