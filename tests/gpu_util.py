"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

from oracle import tsr_oracle as orc


def rel_fro(a, b) -> float:
    a = orc.f64(a); b = orc.f64(b)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def projector_err(X_gpu, X_ref) -> float:
    """|| X X^T - Y Y^T ||_F / || Y Y^T ||_F computed through the small r x r products."""
    X = orc.f64(X_gpu); Y = orc.f64(X_ref)
    # ||XX^T - YY^T||^2 = ||X^T X||^2 + ||Y^T Y||^2 - 2 ||X^T Y||^2
    a = np.linalg.norm(X.T @ X) ** 2; b = np.linalg.norm(Y.T @ Y) ** 2; c = np.linalg.norm(X.T @ Y) ** 2
    return float(np.sqrt(max(a + b - 2 * c, 0.0)) / np.sqrt(b))


def dev(x: torch.Tensor) -> torch.Tensor:
    return x.to("cuda").contiguous()


def padded(x: torch.Tensor, ld: int) -> torch.Tensor:
    """Copy of the 2-D tensor x on the GPU with leading dimension ld (a view into a wider buffer)."""
    m, n = x.shape
    buf = torch.zeros((m, ld), dtype=x.dtype, device="cuda")
    buf[:, :n] = x.to("cuda")
    return buf[:, :n]


def f32(x: float) -> float:
    """The value the C ABI receives for a float argument (hyper-parameters are inputs: the
    oracle gets exactly what the GPU gets)."""
    return float(np.float32(x))


B1, B2, EPS = f32(0.9), f32(0.999), f32(1e-8)
