"""Helpers shared by the GPU parity tests (no method arithmetic)."""
import numpy as np
import torch


def to_np(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> host NumPy; bf16 is widened exactly to float32."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        t = t.to(torch.float32)
    return t.numpy()


def bits(t: torch.Tensor) -> np.ndarray:
    """Raw storage bits of a tensor for memcmp-style comparisons."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy()
    if t.dtype == torch.float32:
        return t.view(torch.int32).numpy()
    return t.numpy()


def rel_err(got: np.ndarray, want: np.ndarray) -> float:
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    denom = np.maximum(np.abs(want), np.finfo(np.float64).tiny)
    return float(np.max(np.abs(got - want) / denom)) if want.size else 0.0


def tol_for(dtype: torch.dtype) -> float:
    """Relative tolerance of norms and scores against the float64 oracle."""
    return 1e-5 if dtype == torch.float32 else 1e-2
