"""Helpers shared by the GPU parity tests: upload of generated tensors, the error
metric, and construction of (raw / packed) factor pairs."""
import numpy as np

import synth_inputs as si

from paper_2604_17709_amd import TOKEN_TILE_BOTH  # noqa: F401  (importing the binding loads nothing)

# bf16 and fp32: the stated bars; fp16: the bf16 bar scaled by the ratio of the unit roundoffs (2^-11 / 2^-8), rounded up
TOL = {"bf16": 1e-2, "f16": 2e-3, "f32": 1e-5}


def to_dev(t: si.Tensor):
    import torch
    if t.dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(t.bits)).cuda()
    return torch.from_numpy(np.ascontiguousarray(t.bits).view(np.int16)).cuda().view(torch.float16 if t.dtype == "f16" else torch.bfloat16)


def to_host(y) -> np.ndarray:
    """Device result -> float64 numpy (exact for f32 and bf16)."""
    import torch
    return y.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def max_err(y: np.ndarray, ref: np.ndarray) -> float:
    """max |y - ref| / max |ref| over one output tensor (the parity gate)."""
    denom = float(np.max(np.abs(ref))) if ref.size else 1.0
    if denom == 0.0:
        return float(np.max(np.abs(y))) if y.size else 0.0
    return float(np.max(np.abs(y - ref))) / denom


def pair(dn, U: si.Tensor, V: si.Tensor, packed: bool):
    """Returns (Pair, keepalive)."""
    Ud, Vd = to_dev(U), to_dev(V)
    p = dn.raw_pair(Ud, Vd)
    if packed:
        return dn.deinfer_pack_factors(p), (Ud, Vd)
    return p, (Ud, Vd)
