"""Helpers shared by the GPU parity tests: upload, error metric, oracle-side references."""
import numpy as np
import torch


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def scaled_error(y: np.ndarray, y_ref: np.ndarray, row_norms: np.ndarray, x: np.ndarray) -> float:
    """max_n |y_n - y*_n| / (||What[n,:]||_2 ||x||_2) for a vector x, or
    max_{m,n} |Y - Y*| / (||What[n,:]||_2 ||X[m,:]||_2) for a matrix X [M,K] and Y [M,N]."""
    x64 = x.astype(np.float64)
    if x.ndim == 1:
        den = row_norms * np.linalg.norm(x64)
    else:
        den = np.linalg.norm(x64, axis=1)[:, None] * row_norms[None, :]
    den = np.where(den == 0, 1.0, den)
    return float(np.max(np.abs(y.astype(np.float64) - y_ref) / den))
