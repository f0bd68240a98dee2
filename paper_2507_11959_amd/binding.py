"""Thin ctypes binding of the potq C ABI (include/potq.h).

Argument marshalling only: every function takes torch CUDA(HIP) tensors, checks
dtype / shape / device / contiguity, and passes raw device pointers plus the
current HIP stream to the shared library.  All computation happens in the
library's kernels.  There is no CPU fallback: if the library has not been
built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import torch  # loads the process's HIP runtime before libpotq.so is opened

from .build import LIB_PATH

LAYOUT_CANONICAL = 0
LAYOUT_TILE16 = 1

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()' "
        "or python paper_2507_11959_amd/build.py). There is no fallback path."
    )

_lib = ctypes.CDLL(LIB_PATH)
_vp, _i64, _int = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int

EXPORTS = {
    "potq_version": (_int, []),
    "potq_strerror": (ctypes.c_char_p, [_int]),
    "potq_packed_row_bytes": (ctypes.c_size_t, [_i64, _int]),
    "potq_packed_bytes": (ctypes.c_size_t, [_i64, _i64, _int]),
    "pot_dequant": (_int, [_vp, _vp, _vp, _i64, _i64, _int, _int, _vp]),
    "int_dequant": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _int, _int, _vp]),
    "pot_dequant_batch": (_int, [_vp, _int, _int, _int, _vp]),
    "int_dequant_batch": (_int, [_vp, _int, _int, _int, _vp]),
    "potq_repack": (_int, [_vp, _vp, _i64, _i64, _int, _int, _vp]),
    "pot_gemv_batch": (_int, [_vp, _int, _vp, _i64, _int, _int, _int, _vp]),
    "int_gemv_batch": (_int, [_vp, _int, _vp, _i64, _int, _int, _int, _vp]),
    "pot_gemv": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _int, _int, _int, _vp]),
    "int_gemv": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _int, _int, _int, _vp]),
    "potq_gemm_workspace_bytes": (ctypes.c_size_t, [_i64, _i64, _i64, _int]),
    "potq_gemv_exponent_form": (_int, [_i64, _i64, _int]),
    "potq_gemv_batch_exponent_form": (_int, [_int, _i64, _int]),
    "pot_gemm": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _int, _vp, ctypes.c_size_t, _vp]),
    "pot_gemm_noalloc": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _int, _vp]),
    "int_gemm": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _int, _int, _int, _vp, ctypes.c_size_t, _vp]),
    "pot_check_scales": (_int, [_vp, _i64, _int, _vp, _vp]),
    "pot_quantize": (_int, [_vp, _vp, _vp, _i64, _i64, _int, _int, _vp]),
    "pot_fakequant_forward": (_int, [_vp, _vp, _vp, _vp, _i64, _i64, _int, _int, _vp]),
    "pot_fakequant_backward": (_int, [_vp, _vp, _vp, _vp, _vp, _i64, _i64, _int, _int, _vp]),
}
for _name, (_res, _args) in EXPORTS.items():
    _f = getattr(_lib, _name)
    _f.restype = _res
    _f.argtypes = _args


class PotqError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"potq status {status}: {_lib.potq_strerror(status).decode()}")


def _ok(status: int) -> None:
    if status != 0:
        raise PotqError(status)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def version() -> int:
    return _lib.potq_version()


def strerror(status: int) -> str:
    return _lib.potq_strerror(status).decode()


def packed_row_bytes(K: int, bits: int) -> int:
    return _lib.potq_packed_row_bytes(K, bits)


def packed_bytes(N: int, K: int, bits: int) -> int:
    return _lib.potq_packed_bytes(N, K, bits)


def _shape_codes(codes: torch.Tensor, K: int, bits: int) -> int:
    n_bytes = codes.numel() * codes.element_size()
    rb = packed_row_bytes(K, bits)
    if rb == 0 or n_bytes % rb:
        raise ValueError("codes size is not a whole number of packed rows")
    return n_bytes // rb


def _per_group(t: torch.Tensor, N: int, K: int, group: int, name: str) -> None:
    """One value per (row, group): a wrong group size or a short tensor must not reach the kernels."""
    if group not in (64, 128):
        raise ValueError("group must be 64 or 128")
    if t.numel() != N * (K // group):
        raise ValueError(f"{name} must hold N*(K/group) = {N * (K // group)} values, got {t.numel()}")


def _numel(t: torch.Tensor, n: int, name: str) -> None:
    if t.numel() != n:
        raise ValueError(f"{name} must hold {n} values, got {t.numel()}")


def pot_dequant(codes, scales, K: int, bits: int, group: int = 128, out=None):
    """codes: uint8 (N, K*bits/8) canonical; scales: fp16 (N, K/group) -> fp16 (N, K)."""
    N = _shape_codes(codes, K, bits)
    _per_group(scales, N, K, group, "scales")
    if out is None:
        out = torch.empty((N, K), dtype=torch.float16, device=codes.device)
    _numel(out, N * K, "out")
    _ok(_lib.pot_dequant(_dev(codes, torch.uint8, "codes"), _dev(scales, torch.float16, "scales"),
                         _dev(out, torch.float16, "out"), N, K, bits, group, _stream()))
    return out


def int_dequant(codes, scales, zeros, K: int, bits: int, group: int = 128, out=None):
    N = _shape_codes(codes, K, bits)
    _per_group(scales, N, K, group, "scales")
    _per_group(zeros, N, K, group, "zeros")
    if out is None:
        out = torch.empty((N, K), dtype=torch.float16, device=codes.device)
    _numel(out, N * K, "out")
    _ok(_lib.int_dequant(_dev(codes, torch.uint8, "codes"), _dev(scales, torch.float16, "scales"),
                         _dev(zeros, torch.float16, "zeros"), _dev(out, torch.float16, "out"),
                         N, K, bits, group, _stream()))
    return out


MAX_BATCH = 16


class DequantItem(ctypes.Structure):
    """Mirror of `potq_dequant_item`."""
    _fields_ = [("codes", _vp), ("scales", _vp), ("zeros", _vp), ("out_f16", _vp), ("N", _i64), ("K", _i64)]


def make_batch(mats, is_int: bool = False, group: int = 128):
    """mats: list of (codes, scales, zeros-or-None, out, K, bits) device tensors -> ctypes descriptor array.

    The returned array only holds raw pointers: keep the tensors alive while it is in use."""
    arr = (DequantItem * len(mats))()
    for i, (codes, scales, zeros, out, K, bits) in enumerate(mats):
        N = _shape_codes(codes, K, bits)
        _per_group(scales, N, K, group, "scales")
        if is_int:
            _per_group(zeros, N, K, group, "zeros")
        _numel(out, N * K, "out")
        arr[i].codes = _dev(codes, torch.uint8, "codes")
        arr[i].scales = _dev(scales, torch.float16, "scales")
        arr[i].zeros = _dev(zeros, torch.float16, "zeros") if is_int else None
        arr[i].out_f16 = _dev(out, torch.float16, "out")
        arr[i].N, arr[i].K = N, K
    return arr


def pot_dequant_batch(mats, bits: int, group: int = 128):
    """mats: list of (codes, scales, out, K); one launch for all of them."""
    arr = make_batch([(c, s, None, o, K, bits) for (c, s, o, K) in mats], group=group)
    _ok(_lib.pot_dequant_batch(arr, len(mats), bits, group, _stream()))


def int_dequant_batch(mats, bits: int, group: int = 128):
    """mats: list of (codes, scales, zeros, out, K); one launch for all of them."""
    arr = make_batch([(c, s, z, o, K, bits) for (c, s, z, o, K) in mats], is_int=True, group=group)
    _ok(_lib.int_dequant_batch(arr, len(mats), bits, group, _stream()))


def potq_repack(src, K: int, bits: int, to_layout: int = LAYOUT_TILE16, out=None):
    N = _shape_codes(src, K, bits)
    if out is None:
        out = torch.empty_like(src)
    _numel(out, src.numel(), "dst")
    _ok(_lib.potq_repack(_dev(src, torch.uint8, "src"), _dev(out, torch.uint8, "dst"), N, K, bits, to_layout,
                         _stream()))
    return out


def pot_gemv(codes, scales, x, K: int, bits: int, group: int = 128, layout: int = LAYOUT_TILE16, out=None):
    N = _shape_codes(codes, K, bits)
    if x.numel() != K:
        raise ValueError("x must have K elements")
    _per_group(scales, N, K, group, "scales")
    if out is None:
        out = torch.empty((N,), dtype=torch.float16, device=codes.device)
    _numel(out, N, "y")
    _ok(_lib.pot_gemv(_dev(codes, torch.uint8, "codes"), _dev(scales, torch.float16, "scales"),
                      _dev(x, torch.float16, "x"), _dev(out, torch.float16, "y"), N, K, bits, group, layout,
                      _stream()))
    return out


def int_gemv(codes, scales, zeros, x, K: int, bits: int, group: int = 128, layout: int = LAYOUT_TILE16, out=None):
    N = _shape_codes(codes, K, bits)
    if x.numel() != K:
        raise ValueError("x must have K elements")
    _per_group(scales, N, K, group, "scales")
    _per_group(zeros, N, K, group, "zeros")
    if out is None:
        out = torch.empty((N,), dtype=torch.float16, device=codes.device)
    _numel(out, N, "y")
    _ok(_lib.int_gemv(_dev(codes, torch.uint8, "codes"), _dev(scales, torch.float16, "scales"),
                      _dev(zeros, torch.float16, "zeros"), _dev(x, torch.float16, "x"),
                      _dev(out, torch.float16, "y"), N, K, bits, group, layout, _stream()))
    return out


def gemm_workspace(M: int, N: int, K: int, bits: int, device="cuda:0"):
    """A workspace tensor of the size potq_gemm_workspace_bytes() asks for (None if it asks for nothing)."""
    n = _lib.potq_gemm_workspace_bytes(M, N, K, bits)
    return torch.empty((n,), dtype=torch.uint8, device=device) if n else None


def _ws(workspace):
    if workspace is None:
        return None, 0
    return _dev(workspace, torch.uint8, "workspace"), workspace.numel()


class GemvItem(ctypes.Structure):
    """Mirror of `potq_gemv_item`."""
    _fields_ = [("codes", _vp), ("scales", _vp), ("zeros", _vp), ("y_f16", _vp), ("N", _i64)]


def make_gemv_batch(mats, K: int, bits: int, is_int: bool = False, group: int = 128):
    """mats: list of (codes, scales, zeros-or-None, y) device tensors -> ctypes descriptor array (raw pointers)."""
    arr = (GemvItem * len(mats))()
    for i, (codes, scales, zeros, y) in enumerate(mats):
        N = _shape_codes(codes, K, bits)
        _per_group(scales, N, K, group, "scales")
        if is_int:
            _per_group(zeros, N, K, group, "zeros")
        _numel(y, N, "y")
        arr[i].codes = _dev(codes, torch.uint8, "codes")
        arr[i].scales = _dev(scales, torch.float16, "scales")
        arr[i].zeros = _dev(zeros, torch.float16, "zeros") if is_int else None
        arr[i].y_f16 = _dev(y, torch.float16, "y")
        arr[i].N = _shape_codes(codes, K, bits)
    return arr


def potq_gemv_exponent_form(N: int, K: int, bits: int) -> bool:
    """Whether pot_gemv serves an N x K matrix in the exponent form."""
    return bool(_lib.potq_gemv_exponent_form(N, K, bits))


def potq_gemv_batch_exponent_form(count: int, K: int, bits: int) -> bool:
    """Whether pot_gemv_batch serves `count` matrices of row length K in the exponent form."""
    return bool(_lib.potq_gemv_batch_exponent_form(count, K, bits))


def pot_gemv_batch(mats, x, K: int, bits: int, group: int = 128, layout: int = LAYOUT_TILE16):
    """mats: list of (codes, scales) sharing x; -> list of y tensors, one launch."""
    ys = [torch.empty((_shape_codes(c, K, bits),), dtype=torch.float16, device=c.device) for (c, s) in mats]
    if x.numel() != K:
        raise ValueError("x must have K elements")
    arr = make_gemv_batch([(c, s, None, y) for (c, s), y in zip(mats, ys)], K, bits, group=group)
    _ok(_lib.pot_gemv_batch(arr, len(mats), _dev(x, torch.float16, "x"), K, bits, group, layout, _stream()))
    return ys


def int_gemv_batch(mats, x, K: int, bits: int, group: int = 128, layout: int = LAYOUT_TILE16):
    """mats: list of (codes, scales, zeros) sharing x; -> list of y tensors, one launch."""
    ys = [torch.empty((_shape_codes(c, K, bits),), dtype=torch.float16, device=c.device) for (c, s, z) in mats]
    if x.numel() != K:
        raise ValueError("x must have K elements")
    arr = make_gemv_batch([(c, s, z, y) for (c, s, z), y in zip(mats, ys)], K, bits, is_int=True, group=group)
    _ok(_lib.int_gemv_batch(arr, len(mats), _dev(x, torch.float16, "x"), K, bits, group, layout, _stream()))
    return ys


def pot_gemm(codes, scales, X, K: int, bits: int, group: int = 128, layout: int = LAYOUT_TILE16, out=None,
             workspace=None):
    N = _shape_codes(codes, K, bits)
    if X.dim() != 2 or X.shape[1] != K:
        raise ValueError("X must be (M, K)")
    M = X.shape[0]
    _per_group(scales, N, K, group, "scales")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=codes.device)
    _numel(out, M * N, "Y")
    wp, wn = _ws(workspace)
    _ok(_lib.pot_gemm(_dev(codes, torch.uint8, "codes"), _dev(scales, torch.float16, "scales"),
                      _dev(X, torch.float16, "X"), _dev(out, torch.float16, "Y"), M, N, K, bits, group, layout,
                      wp, wn, _stream()))
    return out


def pot_gemm_noalloc(codes, scales, X, out, K: int, bits: int, group: int = 128, layout: int = LAYOUT_TILE16):
    """pot_gemm with the library's built-in scratch buffer; `out` (M, N) is the caller's: nothing is allocated."""
    N = _shape_codes(codes, K, bits)
    if X.dim() != 2 or X.shape[1] != K:
        raise ValueError("X must be (M, K)")
    M = X.shape[0]
    if tuple(out.shape) != (M, N):
        raise ValueError("out must be (M, N)")
    _per_group(scales, N, K, group, "scales")
    _ok(_lib.pot_gemm_noalloc(_dev(codes, torch.uint8, "codes"), _dev(scales, torch.float16, "scales"),
                              _dev(X, torch.float16, "X"), _dev(out, torch.float16, "Y"), M, N, K, bits, group,
                              layout, _stream()))
    return out


def int_gemm(codes, scales, zeros, X, K: int, bits: int, group: int = 128, layout: int = LAYOUT_TILE16, out=None,
             workspace=None):
    N = _shape_codes(codes, K, bits)
    if X.dim() != 2 or X.shape[1] != K:
        raise ValueError("X must be (M, K)")
    M = X.shape[0]
    _per_group(scales, N, K, group, "scales")
    _per_group(zeros, N, K, group, "zeros")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=codes.device)
    _numel(out, M * N, "Y")
    wp, wn = _ws(workspace)
    _ok(_lib.int_gemm(_dev(codes, torch.uint8, "codes"), _dev(scales, torch.float16, "scales"),
                      _dev(zeros, torch.float16, "zeros"), _dev(X, torch.float16, "X"),
                      _dev(out, torch.float16, "Y"), M, N, K, bits, group, layout, wp, wn, _stream()))
    return out


def pot_quantize(W, bits: int, group: int = 128):
    """W: fp16 (N, K) -> (packed codes uint8 (N, K*bits/8) canonical, scales fp16 (N, K/group))."""
    if W.dim() != 2:
        raise ValueError("W must be (N, K)")
    N, K = W.shape
    codes = torch.empty((N, K * bits // 8), dtype=torch.uint8, device=W.device)
    scales = torch.empty((N, K // group), dtype=torch.float16, device=W.device)
    _ok(_lib.pot_quantize(_dev(W, torch.float16, "W"), _dev(codes, torch.uint8, "codes"),
                          _dev(scales, torch.float16, "scales"), N, K, bits, group, _stream()))
    return codes, scales


def pot_fakequant_forward(W, S, Gamma, bits: int, group: int = 128):
    """Step 2 forward: W fp16 (N, K), S fp16 (N, K/group), Gamma float32 (N, K/group) -> w~ fp16 (N, K)."""
    if W.dim() != 2:
        raise ValueError("W must be (N, K)")
    N, K = W.shape
    if tuple(S.shape) != (N, K // group) or tuple(Gamma.shape) != tuple(S.shape):
        raise ValueError("S and Gamma must be (N, K/group)")
    Wq = torch.empty_like(W)
    _ok(_lib.pot_fakequant_forward(_dev(W, torch.float16, "W"), _dev(S, torch.float16, "S"),
                                   _dev(Gamma, torch.float32, "Gamma"), _dev(Wq, torch.float16, "Wq"),
                                   N, K, bits, group, _stream()))
    return Wq


def pot_fakequant_backward(W, S, Gamma, dWq, bits: int, group: int = 128):
    """Step 2 backward (straight-through estimator): dWq fp16 (N, K) -> dL/dGamma float32 (N, K/group)."""
    if W.dim() != 2 or tuple(dWq.shape) != tuple(W.shape):
        raise ValueError("W and dWq must be (N, K)")
    N, K = W.shape
    if tuple(S.shape) != (N, K // group) or tuple(Gamma.shape) != tuple(S.shape):
        raise ValueError("S and Gamma must be (N, K/group)")
    dGamma = torch.empty_like(Gamma)
    _ok(_lib.pot_fakequant_backward(_dev(W, torch.float16, "W"), _dev(S, torch.float16, "S"),
                                    _dev(Gamma, torch.float32, "Gamma"), _dev(dWq, torch.float16, "dWq"),
                                    _dev(dGamma, torch.float32, "dGamma"), N, K, bits, group, _stream()))
    return dGamma


def pot_check_scales(scales, bits: int) -> int:
    """Number of scales outside the exact domain (copies one int64 back: synchronises)."""
    bad = torch.empty((1,), dtype=torch.int64, device=scales.device)
    _ok(_lib.pot_check_scales(_dev(scales, torch.float16, "scales"), scales.numel(), bits, bad.data_ptr(), _stream()))
    return int(bad.item())


def raw():
    """The ctypes library object, for tests that call the ABI with hand-made arguments."""
    return _lib
