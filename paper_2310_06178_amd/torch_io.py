"""Moving numpy inputs to the GPU and results back (plumbing only, no arithmetic).

bf16 travels as uint16 bit patterns on the numpy side (numpy has no bf16)."""
from __future__ import annotations

import numpy as np
import torch

TORCH_DTYPE = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16,
               "i8": torch.int8, "i32": torch.int32}


def to_device(a: np.ndarray | None, kind: str, device="cuda:0"):
    """kind: 'codes', 'scales', or an activation dtype name ('f32','f16','bf16','i8')."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if kind == "codes":
        assert a.dtype == np.uint8
        return torch.from_numpy(a).to(device)
    if kind == "scales":
        assert a.dtype == np.float16
        return torch.from_numpy(a).to(device)
    if kind == "bf16":
        assert a.dtype == np.uint16
        return torch.from_numpy(a.view(np.int16)).to(device).view(torch.bfloat16)
    want = {"f32": np.float32, "f16": np.float16, "i8": np.int8}[kind]
    assert a.dtype == want, (a.dtype, want)
    return torch.from_numpy(a).to(device)


def empty_output(b: int, m: int, y_dtype: str, device="cuda:0", ldy: int | None = None):
    ldy = m if ldy is None else ldy
    return torch.empty((b, ldy), dtype=TORCH_DTYPE[y_dtype], device=device)


def to_host(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> numpy; bf16 comes back as uint16 bit patterns."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of host results (uint16 = bf16 bits) to fp64."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)
