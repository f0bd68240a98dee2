"""A second, independent statement of the path in vectorised numpy.

Used only by the CPU tests as a cross-check of the C oracle: it relies on
numpy's own float16 type, ``np.unpackbits`` and ``np.ldexp`` instead of the
oracle's software conversions and bit loops, so the two can only agree if both
are right.  Citations: Sec. 3.1 Eq. (1)-(5), Sec. 4.1 Eq. (9)-(11), Sec. 4.2.
"""
import numpy as np


def unpack(packed: np.ndarray, K: int, bits: int) -> np.ndarray:
    """(N, K*bits/8) uint8 little-endian bit stream -> (N, K) integer codes."""
    N = packed.shape[0]
    stream = np.unpackbits(packed, axis=1, bitorder="little")[:, : K * bits]
    fields = stream.reshape(N, K, bits).astype(np.uint8)
    weights = (1 << np.arange(bits)).astype(np.uint8)
    return (fields * weights).sum(axis=2).astype(np.uint8)


def pack(codes: np.ndarray, bits: int) -> np.ndarray:
    N, K = codes.shape
    fields = (codes[:, :, None] >> np.arange(bits)[None, None, :]) & 1
    return np.packbits(fields.reshape(N, K * bits).astype(np.uint8), axis=1, bitorder="little")


def pot_dequant(packed, scales_f16, K, bits, group) -> np.ndarray:
    """-> (N, K) float16, by the definition (-1)^sign * 2^E * s."""
    c = unpack(packed, K, bits)
    sign = (c >> (bits - 1)) & 1
    E = (c & ((1 << (bits - 1)) - 1)).astype(np.int32)
    s = np.repeat(scales_f16.astype(np.float16), group, axis=1)
    with np.errstate(over="ignore"):
        mag = np.ldexp(s, E)            # float16 ldexp: exact or IEEE-rounded
    return np.where(sign == 1, -mag, mag).astype(np.float16)


def int_dequant(packed, S_f16, Z_f16, K, bits, group) -> np.ndarray:
    c = unpack(packed, K, bits).astype(np.float64)
    S = np.repeat(S_f16.astype(np.float64), group, axis=1)
    Z = np.repeat(Z_f16.astype(np.float64), group, axis=1)
    return ((c + Z) * S).astype(np.float16)   # exact product in float64, one rounding


def gemm_f64(W_f16: np.ndarray, X_f16: np.ndarray) -> np.ndarray:
    """X (M,K) . W~^T (K,N) in float64 (library matmul)."""
    return X_f16.astype(np.float64) @ W_f16.astype(np.float64).T
