"""Helpers for the GPU parity tests (host <-> device copies, the error measure)."""
import numpy as np
import torch

DEV = "cuda:0"

# Tolerance of the fused GEMV / GEMM against the oracle: element-wise relative
# error with the denominator floored at 2^-10 of the output's rms value.
REL_TOL = 2e-3


def dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.float16)
    return torch.from_numpy(a).to(DEV)


def host_bits(t: torch.Tensor) -> np.ndarray:
    """fp16 tensor -> uint16 bit patterns on the host."""
    return t.detach().cpu().numpy().view(np.uint16)


def rel_err(y_bits: np.ndarray, ref_bits: np.ndarray):
    """(max element-wise relative error with floored denominator, normwise error, #elements on the floor)."""
    y = y_bits.view(np.float16).astype(np.float64).ravel()
    r = ref_bits.view(np.float16).astype(np.float64).ravel()
    rms = np.sqrt(np.mean(r * r)) if r.size else 0.0
    floor = rms * 2.0 ** -10
    den = np.maximum(np.abs(r), floor)
    den = np.where(den == 0.0, 1.0, den)
    err = np.abs(y - r) / den
    normwise = np.abs(y - r).max() / max(np.abs(r).max(), 1e-300) if r.size else 0.0
    return (err.max() if r.size else 0.0), normwise, int((np.abs(r) < floor).sum())
