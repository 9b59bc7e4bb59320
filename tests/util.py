"""Helpers shared by the GPU parity tests (no method arithmetic of the product path)."""
import numpy as np
import torch

import workloads as wl


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    """Round a float64/float32 host array to the call dtype and upload it."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.cuda().contiguous()


def to_host(t: torch.Tensor) -> np.ndarray:
    """Download as float64 (exact for both storage types)."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_fro(a: np.ndarray, ref: np.ndarray) -> float:
    return float(np.linalg.norm((a - ref).ravel()) / max(np.linalg.norm(ref.ravel()), 1e-300))


def sin_theta(Ua: np.ndarray, Ub: np.ndarray) -> float:
    """sine of the largest principal angle between span(Ua) and span(Ub), Ua orthonormal."""
    return float(np.linalg.norm(Ub - Ua @ (Ua.T @ Ub), 2))


def tol(dtype: str) -> float:
    return 1e-2 if dtype == "bf16" else 1e-4


def torch_dtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32
