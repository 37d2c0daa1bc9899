"""Helpers shared by the GPU parity tests (comparison metrics, host copies)."""
import numpy as np
import torch

TOL_F32 = 1e-5     # relative Frobenius error, fp32 path
TOL_BF16 = 3e-3    # relative Frobenius error, bf16 matrix-core path
TOL_S = 2e-6       # relative, per element of s


def to_np64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def rel_fro(a: np.ndarray, ref: np.ndarray) -> float:
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(a - ref) / den) if den > 0 else float(np.linalg.norm(a))


def upper(a: np.ndarray) -> np.ndarray:
    """Entries on or above the diagonal of the last two axes (others zeroed)."""
    return np.triu(a)


def say(msg: str) -> None:
    print(msg, flush=True)
