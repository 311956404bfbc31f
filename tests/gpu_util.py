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


def critical_column_plan(K: int, N: int):
    """How many critical columns the tiled GEMM takes as fp16 slabs through its ring, and from how many on it makes
    its dense pass instead (the host-side plan of csrc/gemm.h, restated for the tests that aim at either side)."""
    n_slabs = (K + 127) // 128 * 2
    npad = (N + 255) // 256 * 256
    cols = min(n_slabs * 32, 2048, (96 << 20) // (npad * 2))
    in_slabs = 32 * (8 + cols // 32)
    left = 3.7 * n_slabs - in_slabs * (1.5 / 32)
    return in_slabs, in_slabs + (int(left / 0.44) if left > 0 else 0)
