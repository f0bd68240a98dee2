"""Helpers for the GPU parity tests (host <-> device copies, the error measure)."""
import numpy as np
import torch

DEV = "cuda:0"

# Tolerance of the fused GEMV / GEMM against the oracle: element-wise relative
# error |y - ref| / max(|ref|, delta).  The floor delta keeps an output that
# cancelled to (nearly) zero from turning the absolute noise of fp32
# accumulation into an unbounded relative error: the kernels round once, to
# fp32 (2^-24 relative to the running sum, itself of the size of the output's
# rms value), per 32-product step, K/32 times per output; eight standard
# deviations of that random walk may use up the whole tolerance on the floor,
#     delta = rms(ref) * max(2^-10, 8 * 2^-24 * sqrt(K / 32) / REL_TOL).
REL_TOL = 2e-3


def floor_fraction(K: int) -> float:
    """delta / rms(ref) for a contraction of length K."""
    return max(2.0 ** -10, 8.0 * 2.0 ** -24 * (K / 32.0) ** 0.5 / REL_TOL)


def dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.float16)
    return torch.from_numpy(a).to(DEV)


def host_bits(t: torch.Tensor) -> np.ndarray:
    """fp16 tensor -> uint16 bit patterns on the host."""
    return t.detach().cpu().numpy().view(np.uint16)


def rel_err(y_bits: np.ndarray, ref_bits: np.ndarray, K: int):
    """(max element-wise relative error with floored denominator, normwise error, #elements on the floor)."""
    y = y_bits.view(np.float16).astype(np.float64).ravel()
    r = ref_bits.view(np.float16).astype(np.float64).ravel()
    rms = np.sqrt(np.mean(r * r)) if r.size else 0.0
    floor = rms * floor_fraction(K)
    den = np.maximum(np.abs(r), floor)
    den = np.where(den == 0.0, 1.0, den)
    err = np.abs(y - r) / den
    normwise = np.abs(y - r).max() / max(np.abs(r).max(), 1e-300) if r.size else 0.0
    return (err.max() if r.size else 0.0), normwise, int((np.abs(r) < floor).sum())


GUARD_BYTES = 4096
GUARD_PATTERN = 0xA5


class Guarded:
    """An output tensor with a band of GUARD_BYTES pattern bytes on either side in the same allocation:
    an entry point that writes outside the tensor it was given changes a band."""

    def __init__(self, shape, dtype, fill=None):
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        pad = (-n) % 16
        self.raw = torch.full((GUARD_BYTES + n + pad + GUARD_BYTES,), GUARD_PATTERN, dtype=torch.uint8, device=DEV)
        self.nbytes = n
        self.tensor = self.raw[GUARD_BYTES:GUARD_BYTES + n].view(dtype).reshape(shape)
        if fill is not None:
            self.tensor.fill_(fill)

    def intact(self) -> bool:
        lo = self.raw[:GUARD_BYTES]
        hi = self.raw[GUARD_BYTES + self.nbytes:]
        return bool((lo == GUARD_PATTERN).all()) and bool((hi == GUARD_PATTERN).all())
