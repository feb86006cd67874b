"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

PER_ROUND_TOL = 1e-5      # fp32, one round, max |x-y| / max |y| per tensor
HUNDRED_ROUND_TOL = 1e-4  # after 100 free-running rounds


def normwise(x: np.ndarray, y: np.ndarray) -> float:
    """max_j |x_j - y_j| / max_j |y_j| over the finite entries of the reference y
    (NaN padding must be NaN in both)."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    pad = np.isnan(y)
    assert np.array_equal(np.isnan(x), pad), "padding / validity pattern differs"
    if pad.all():
        return 0.0
    scale = np.abs(y[~pad]).max()
    diff = np.abs(x[~pad] - y[~pad]).max()
    return float(diff / scale) if scale > 0 else float(diff)


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()
