"""Helpers shared by the GPU parity tests: host <-> device conversion and error metrics."""
import numpy as np
import torch

from paper_2511_17560_amd import api


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    """Storage-exact float array -> device tensor of the storage type."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(api.torch_dtype(dtype)).cuda().contiguous()


def idev(x) -> torch.Tensor:
    return torch.as_tensor(np.ascontiguousarray(x, dtype=np.int32), device="cuda")


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def max_elem_rel(got: np.ndarray, want: np.ndarray, floor: float = 1e-3) -> float:
    """Worst element-wise relative error, max |a - b| / max(|b|, floor * max |b|): an element is measured against
    its own size, down to a floor of one thousandth of the tensor's largest entry."""
    want = np.asarray(want, dtype=np.float64)
    assert np.shape(got) == want.shape, (np.shape(got), want.shape)
    if want.size == 0:                 # nothing selected (ratio 0) or nothing left stale (ratio 1)
        return 0.0
    scale = float(np.abs(want).max())
    if scale == 0.0:
        return float(np.abs(got - want).max())
    return float((np.abs(got - want) / np.maximum(np.abs(want), floor * scale)).max())


def max_abs_rel(got: np.ndarray, want: np.ndarray) -> float:
    """max |a - b| / max |b| over the tensor."""
    assert np.shape(got) == np.shape(want), (np.shape(got), np.shape(want))
    if np.size(want) == 0:
        return 0.0
    denom = float(np.abs(want).max())
    return float(np.abs(got - want).max()) / (denom if denom > 0 else 1.0)
