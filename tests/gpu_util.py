"""Helpers shared by the GPU parity tests: move seeded numpy inputs to the device, run the HIP
layer, and the error metric of the parity bar."""
import numpy as np
import torch

DEV = "cuda:0"


def to_dev(a: np.ndarray, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def to_np(t: torch.Tensor) -> np.ndarray:
    torch.cuda.synchronize()
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy().astype(np.float64)
    if t.dtype == torch.float32:
        return t.cpu().numpy().astype(np.float64)
    return t.cpu().numpy()


def max_norm_err(got, ref) -> float:
    """max|got - ref| / max|ref|  (the tensor-level relative error of the parity bar)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.abs(ref).max()
    if den == 0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / den)


def torch_dtype(name: str):
    return torch.float32 if name == "f32" else torch.bfloat16
