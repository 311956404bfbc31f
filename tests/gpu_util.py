"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch


def to_gpu(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def assert_y_close(y_gpu: np.ndarray, y_ref: np.ndarray, rel: float = 1e-2):
    """The fp16 output bar: relative Frobenius error <= rel and, element by element,
    |delta| <= rel * |ref| + rel * rms(ref).  Returns the observed worst ratios."""
    g = y_gpu.astype(np.float64)
    r = y_ref.astype(np.float64)
    assert g.shape == r.shape
    assert np.all(np.isfinite(g))
    if r.size == 0:
        return 0.0, 0.0
    fro = np.linalg.norm(g - r) / max(np.linalg.norm(r), 1e-30)
    rms = np.sqrt(np.mean(r * r))
    bound = rel * np.abs(r) + rel * rms
    worst = float(np.max(np.abs(g - r) / np.maximum(bound, 1e-30)))
    assert fro <= rel, ("Frobenius", fro)
    assert worst <= 1.0, ("elementwise", worst)
    return fro, worst
