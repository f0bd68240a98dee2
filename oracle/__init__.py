"""ctypes front end of the CPU oracle (oracle/potq_oracle.c).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: only tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg may import this package.  It imports nothing from
the GPU package and the GPU package imports nothing from here.

All arrays are numpy arrays on the host.  fp16 quantities travel as uint16 bit
patterns (or numpy float16 viewed as uint16) so that no conversion other than
the oracle's own is involved.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "potq_oracle.c")
# POTQ_ORACLE_SANITIZE=1 in the environment: the same source built with the undefined-behaviour
# sanitizer (every finding aborts), kept beside the plain build; the CPU test suite re-runs the
# oracle's pins under it (tests/test_oracle_sanitizers.py)
_SANITIZE = os.environ.get("POTQ_ORACLE_SANITIZE", "") not in ("", "0")
_LIB = os.path.join(_HERE, "libpotq_oracle_ubsan.so" if _SANITIZE else "libpotq_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        extra = ["-g", "-fsanitize=undefined", "-fno-sanitize-recover=all"] if _SANITIZE else []
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", *extra,
             "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def _L():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c = ctypes
        lib.orc_half_to_double.restype = c.c_double
        lib.orc_half_to_double.argtypes = [c.c_uint16]
        lib.orc_double_to_half.restype = c.c_uint16
        lib.orc_double_to_half.argtypes = [c.c_double]
        lib.orc_packed_row_bytes.restype = c.c_size_t
        lib.orc_packed_row_bytes.argtypes = [c.c_int64, c.c_int]
        lib.orc_pack_codes.restype = None
        lib.orc_pack_codes.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int]
        lib.orc_unpack_codes.restype = None
        lib.orc_unpack_codes.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int]
        lib.orc_decode_def.restype = c.c_uint16
        lib.orc_decode_def.argtypes = [c.c_uint, c.c_uint16, c.c_int]
        lib.orc_decode_bits.restype = c.c_uint16
        lib.orc_decode_bits.argtypes = [c.c_uint, c.c_uint16, c.c_int]
        lib.orc_int_decode.restype = c.c_uint16
        lib.orc_int_decode.argtypes = [c.c_uint, c.c_uint16, c.c_uint16]
        lib.orc_scale_in_domain.restype = c.c_int
        lib.orc_scale_in_domain.argtypes = [c.c_uint16, c.c_int]
        lib.orc_check_scales.restype = c.c_int64
        lib.orc_check_scales.argtypes = [c.c_void_p, c.c_int64, c.c_int]
        lib.orc_pot_dequant.restype = None
        lib.orc_pot_dequant.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64,
                                        c.c_int, c.c_int, c.c_int, c.c_int]
        lib.orc_int_dequant.restype = None
        lib.orc_int_dequant.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64,
                                        c.c_int64, c.c_int, c.c_int, c.c_int]
        lib.orc_gemm.restype = None
        lib.orc_gemm.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
                                 c.c_int64, c.c_int64, c.c_int64, c.c_int, c.c_int, c.c_int]
        lib.orc_pot_quantize.restype = None
        lib.orc_pot_quantize.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64,
                                         c.c_int, c.c_int, c.c_int]
        lib.orc_fakequant_forward.restype = None
        lib.orc_fakequant_forward.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64,
                                              c.c_int, c.c_int, c.c_int]
        lib.orc_fakequant_backward.restype = None
        lib.orc_fakequant_backward.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64,
                                               c.c_int64, c.c_int, c.c_int, c.c_int]
        lib.orc_max_threads.restype = c.c_int
        lib.orc_max_threads.argtypes = []
        _lib = lib
    return _lib


def _u8(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint8, a.dtype
    return a


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def max_threads() -> int:
    return int(_L().orc_max_threads())


def half_to_double(bits: int) -> float:
    return float(_L().orc_half_to_double(int(bits)))


def double_to_half(v: float) -> int:
    return int(_L().orc_double_to_half(float(v)))


def packed_row_bytes(K: int, bits: int) -> int:
    return int(_L().orc_packed_row_bytes(K, bits))


def pack_codes(codes: np.ndarray, bits: int) -> np.ndarray:
    """codes: (N, K) uint8, one code per element -> (N, row_bytes) uint8 bit stream."""
    codes = _u8(codes)
    N, K = codes.shape
    out = np.empty((N, packed_row_bytes(K, bits)), dtype=np.uint8)
    _L().orc_pack_codes(_p(codes), _p(out), N, K, bits)
    return out


def unpack_codes(packed: np.ndarray, K: int, bits: int) -> np.ndarray:
    packed = _u8(packed)
    N = packed.shape[0]
    assert packed.shape[1] == packed_row_bytes(K, bits)
    out = np.empty((N, K), dtype=np.uint8)
    _L().orc_unpack_codes(_p(packed), _p(out), N, K, bits)
    return out


def decode_def(code: int, scale_bits: int, bits: int) -> int:
    return int(_L().orc_decode_def(code, scale_bits, bits))


def decode_bits(code: int, scale_bits: int, bits: int) -> int:
    return int(_L().orc_decode_bits(code, scale_bits, bits))


def int_decode(code: int, scale_bits: int, zero_bits: int) -> int:
    return int(_L().orc_int_decode(code, scale_bits, zero_bits))


def scale_in_domain(scale_bits: int, bits: int) -> bool:
    return bool(_L().orc_scale_in_domain(scale_bits, bits))


def check_scales(scales: np.ndarray, bits: int) -> int:
    s = _u16(scales)
    return int(_L().orc_check_scales(_p(s), s.size, bits))


def pot_dequant(packed, scales, K: int, bits: int, group: int, use_bit_recipe: bool = False,
                nthreads: int = 1) -> np.ndarray:
    """-> (N, K) uint16 bit patterns of the fp16 de-quantised matrix."""
    packed = _u8(packed)
    scales = _u16(scales)
    N = packed.shape[0]
    assert packed.shape[1] == packed_row_bytes(K, bits) and K % group == 0
    assert scales.shape == (N, K // group)
    out = np.empty((N, K), dtype=np.uint16)
    _L().orc_pot_dequant(_p(packed), _p(scales), _p(out), N, K, bits, group, int(use_bit_recipe), nthreads)
    return out


def int_dequant(packed, scales, zeros, K: int, bits: int, group: int, nthreads: int = 1) -> np.ndarray:
    packed = _u8(packed)
    scales = _u16(scales)
    zeros = _u16(zeros)
    N = packed.shape[0]
    assert packed.shape[1] == packed_row_bytes(K, bits) and K % group == 0
    assert scales.shape == (N, K // group) and zeros.shape == scales.shape
    out = np.empty((N, K), dtype=np.uint16)
    _L().orc_int_dequant(_p(packed), _p(scales), _p(zeros), _p(out), N, K, bits, group, nthreads)
    return out


def gemm(packed, scales, zeros, X, K: int, bits: int, group: int, nthreads: int = 1, want_f64: bool = False):
    """Y = X . W~^T.  X: (M, K) fp16 (or uint16 bits); zeros None => PoT.

    -> Y (M, N) uint16 bit patterns [, Y64 (M, N) float64 unrounded sums]."""
    packed = _u8(packed)
    scales = _u16(scales)
    X = _u16(X)
    if X.ndim == 1:
        X = X[None, :]
    M = X.shape[0]
    N = packed.shape[0]
    assert X.shape[1] == K and packed.shape[1] == packed_row_bytes(K, bits) and K % group == 0
    assert scales.shape == (N, K // group)
    zp = None
    if zeros is not None:
        zeros = _u16(zeros)
        assert zeros.shape == scales.shape
        zp = _p(zeros)
    Y = np.empty((M, N), dtype=np.uint16)
    Y64 = np.empty((M, N), dtype=np.float64) if want_f64 else None
    _L().orc_gemm(_p(packed), _p(scales), zp, _p(X), _p(Y), _p(Y64) if want_f64 else None,
                  M, N, K, bits, group, nthreads)
    return (Y, Y64) if want_f64 else Y


def gemv(packed, scales, zeros, x, K: int, bits: int, group: int, nthreads: int = 1, want_f64: bool = False):
    r = gemm(packed, scales, zeros, np.asarray(x).reshape(1, -1), K, bits, group, nthreads, want_f64)
    if want_f64:
        return r[0][0], r[1][0]
    return r[0]


def pot_quantize(W, bits: int, group: int, nthreads: int = 1, want_index: bool = False):
    """Step 1 scale search (Algorithm 1).  W: (N, K) fp16 (or uint16 bits).

    -> codes (N, K) uint8 one code per element, scales (N, K/group) uint16 bits [, best multiplier index]."""
    W = _u16(W)
    N, K = W.shape
    assert K % group == 0
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((N, K // group), dtype=np.uint16)
    idx = np.empty((N, K // group), dtype=np.int32) if want_index else None
    _L().orc_pot_quantize(_p(W), _p(codes), _p(scales), _p(idx) if want_index else None, N, K, bits, group, nthreads)
    return (codes, scales, idx) if want_index else (codes, scales)


def _f32(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float32, a.dtype
    return a


def fakequant_forward(W, S, Gamma, bits: int, group: int, nthreads: int = 1) -> np.ndarray:
    """Step 2 forward (Sec. 3.3): W (N, K) fp16, S (N, K/group) fp16, Gamma (N, K/group) float32
    -> reconstructed weights (N, K) as uint16 bit patterns of fp16."""
    W = _u16(W)
    S = _u16(S)
    Gamma = _f32(Gamma)
    N, K = W.shape
    assert K % group == 0 and S.shape == (N, K // group) and Gamma.shape == S.shape
    out = np.empty((N, K), dtype=np.uint16)
    _L().orc_fakequant_forward(_p(W), _p(S), _p(Gamma), _p(out), N, K, bits, group, nthreads)
    return out


def fakequant_backward(W, S, Gamma, dWq, bits: int, group: int, nthreads: int = 1) -> np.ndarray:
    """Step 2 backward (straight-through estimator): dWq (N, K) fp16 -> dL/dGamma (N, K/group) float32."""
    W = _u16(W)
    S = _u16(S)
    Gamma = _f32(Gamma)
    dWq = _u16(dWq)
    N, K = W.shape
    assert K % group == 0 and S.shape == (N, K // group) and Gamma.shape == S.shape and dWq.shape == W.shape
    out = np.empty((N, K // group), dtype=np.float32)
    _L().orc_fakequant_backward(_p(W), _p(S), _p(Gamma), _p(dWq), _p(out), N, K, bits, group, nthreads)
    return out
