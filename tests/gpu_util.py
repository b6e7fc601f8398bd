"""Helpers for the GPU parity tests: numpy <-> torch marshalling and the error
metric.  (No method arithmetic lives here.)"""
import numpy as np
import torch


def to_dev(a: np.ndarray, pinned=False) -> torch.Tensor:
    """numpy array (float32 / int32 / uint16 bf16 bits) -> torch tensor on the
    GPU (uint16 becomes torch.bfloat16 with the same bits)."""
    if a.dtype == np.uint16:
        t = torch.from_numpy(a.view(np.int16)).view(torch.bfloat16)
    else:
        t = torch.from_numpy(a)
    if pinned:
        p = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
        p.copy_(t)
        return p
    return t.cuda()


def to_host_bits(t: torch.Tensor) -> np.ndarray:
    """GPU tensor -> numpy; bf16 comes back as uint16 bit patterns."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def row_rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max_t ||got[t]-ref[t]||_inf / ||ref[t]||_inf  (rows with ref == 0 must
    match exactly)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.abs(got - ref).max(axis=-1)
    den = np.abs(ref).max(axis=-1)
    zero = den == 0
    if np.any(num[zero] != 0):
        return float("inf")
    return float((num[~zero] / den[~zero]).max()) if (~zero).any() else 0.0


TOL = {"bf16": 2e-2, "f32": 1e-5}
