"""Helpers for the GPU parity tests: bf16 bit patterns <-> device tensors."""
import numpy as np
import torch

import paper_2510_10129_amd as cc

DEV = "cuda:0"


def dev_bf16(bits: np.ndarray) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(DEV)
    return t.view(torch.bfloat16)


def host_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def dev_i32(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def dev_weights(w) -> cc.LayerWeights:
    return cc.LayerWeights(**{k: (None if v is None else dev_bf16(v)) for k, v in w.items()})


def bits_f64(bits):
    return (np.asarray(bits, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def err_stats(got_f64, ref_f64):
    e = np.abs(got_f64 - ref_f64)
    return float(e.max()) if e.size else 0.0, float(e.mean()) if e.size else 0.0
