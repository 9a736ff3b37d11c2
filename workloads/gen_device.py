"""Device-side twins of the host generators, for runs where only speed is
measured and the arrays are too large to draw on the host (a 32-layer stack is
14 GB of weights).  Same shapes and distributions as ``gen``, drawn with
torch's generator on the device; the values differ from the host streams."""
from __future__ import annotations

import torch

from .configs import ModelShape, Workload


def _normal(g, shape, std, mean, device):
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    return (x * std + mean).to(torch.bfloat16)


def layer_weights(model: ModelShape, layer: int, seed: int, device) -> dict:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000 + layer)
    d, f, nq = model.d, model.f, model.n_qkv
    si, so = model.sigma_in, model.sigma_out
    return {
        "w_in_norm": _normal(g, (d,), 0.1, 1.0, device),
        "w_qkv": _normal(g, (nq, d), si, 0.0, device),
        "b_qkv": _normal(g, (nq,), 0.1, 0.0, device) if model.qkv_bias else None,
        "w_o": _normal(g, (d, model.H_q * model.d_h), so, 0.0, device),
        "w_post_norm": _normal(g, (d,), 0.1, 1.0, device),
        "w_gate": _normal(g, (f, d), si, 0.0, device),
        "w_up": _normal(g, (f, d), si, 0.0, device),
        "w_down": _normal(g, (d, f), so, 0.0, device),
    }


def hidden(wl: Workload, device) -> torch.Tensor:
    g = torch.Generator(device=device)
    g.manual_seed(wl.seed * 1000 + 777)
    return _normal(g, (wl.N, wl.model.d), 1.0, 0.0, device)


def cache(wl: Workload, layer: int, device, std: float = 0.6):
    g = torch.Generator(device=device)
    g.manual_seed(wl.seed * 1000 + 500 + layer)
    m = wl.model
    return (_normal(g, (wl.N, m.H_kv, m.d_h), std, 0.0, device),
            _normal(g, (wl.N, m.H_kv, m.d_h), std, 0.0, device))
