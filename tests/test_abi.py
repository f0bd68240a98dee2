"""CPU-only checks of the boundary: the built library loads, exports every
function the public header declares, and rejects bad arguments on the host
(before anything could be launched)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "potq.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2507_11959_amd import binding
    return binding.raw()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_0-9]+)\s*\(", text)
    return sorted({n for n in names if n.startswith(("pot_", "int_", "potq_"))})


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"pot_dequant", "int_dequant", "pot_gemv", "int_gemv", "pot_gemm", "int_gemm", "potq_repack",
            "pot_check_scales", "pot_dequant_batch", "int_dequant_batch", "pot_gemv_batch", "int_gemv_batch", "potq_gemv_batch_exponent_form", "potq_gemm_workspace_bytes", "pot_quantize", "pot_fakequant_forward", "pot_fakequant_backward", "potq_version", "potq_strerror", "potq_packed_row_bytes",
            "potq_packed_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    from paper_2507_11959_amd import binding
    assert set(binding.EXPORTS) == set(names)


def test_sizes_and_strings(lib):
    assert lib.potq_version() >= 100
    assert lib.potq_packed_row_bytes(4096, 3) == 1536
    assert lib.potq_packed_row_bytes(4096, 2) == 1024
    assert lib.potq_packed_bytes(11008, 4096, 2) == 11008 * 1024
    assert lib.potq_packed_row_bytes(100, 3) == 0
    for s in range(9):
        assert lib.potq_strerror(s)
    assert lib.potq_strerror(0) == b"ok"


def test_host_side_validation(lib):
    A, MIS = 0x10000, 0x10004          # fake device addresses: never dereferenced on these paths
    OK, NULL, BITS, GROUP, SHAPE, ALIGN, LAYOUT = 0, 1, 2, 3, 4, 5, 6
    d = lib.pot_dequant
    assert d(None, A, A, 16, 128, 3, 128, None) == NULL
    assert d(A, None, A, 16, 128, 3, 128, None) == NULL
    assert d(A, A, None, 16, 128, 3, 128, None) == NULL
    assert d(A, A, A, 16, 128, 5, 128, None) == BITS
    assert d(A, A, A, 16, 128, 1, 128, None) == BITS
    assert d(A, A, A, 16, 128, 3, 32, None) == GROUP
    assert d(A, A, A, 16, 192, 3, 64, None) == SHAPE
    assert d(A, A, A, -1, 128, 3, 128, None) == SHAPE
    assert d(MIS, A, A, 16, 128, 3, 128, None) == ALIGN
    assert d(A, A, MIS, 16, 128, 3, 128, None) == ALIGN
    assert d(None, None, None, 0, 128, 3, 128, None) == OK          # empty input: nothing to do
    assert d(None, None, None, 16, 0, 2, 64, None) == OK
    i = lib.int_dequant
    assert i(A, A, None, A, 16, 128, 3, 128, None) == NULL
    assert i(A, A, MIS, A, 16, 128, 2, 128, None) == ALIGN
    g = lib.pot_gemv
    assert g(A, A, A, A, 16, 128, 3, 32, 1, None) == GROUP
    assert g(A, A, A, A, 16, 128, 3, 128, 7, None) == LAYOUT
    assert g(A, A, A, A, 8, 128, 3, 128, 1, None) == SHAPE            # tiled layout: N % 16
    assert g(A, A, None, A, 16, 128, 3, 128, 1, None) == NULL
    assert g(A, A, A, None, 16, 128, 3, 128, 1, None) == NULL
    assert g(None, None, None, None, 0, 128, 3, 128, 1, None) == OK
    assert g(A, A, A, A, 16, 76672 + 128, 3, 128, 1, None) == SHAPE   # x no longer fits the LDS of a workgroup
    m = lib.pot_gemm
    assert m(A, A, A, A, -2, 16, 128, 3, 128, 1, None, 0, None) == SHAPE
    assert m(A, A, A, A, 4, 16, 128, 3, 128, 0, None, 0, None) == LAYOUT
    assert m(None, None, None, None, 0, 16, 128, 3, 128, 1, None, 0, None) == OK
    assert m(A, A, A, A, 4, 16, 128, 3, 128, 1, MIS, 1 << 20, None) == ALIGN
    assert lib.int_gemm(A, A, None, A, A, 4, 16, 128, 3, 128, 1, None, 0, None) == NULL
    na = lib.pot_gemm_noalloc                                             # same checks, then the scratch limit
    assert na(A, A, A, A, -2, 16, 128, 3, 128, 1, None) == SHAPE
    assert na(A, A, A, A, 4, 16, 128, 3, 128, 0, None) == LAYOUT
    assert na(A, A, None, A, 4, 16, 128, 3, 128, 1, None) == NULL
    assert na(A, MIS, A, A, 4, 16, 128, 3, 128, 1, None) == ALIGN
    assert na(None, None, None, None, 0, 16, 128, 3, 128, 1, None) == OK
    assert na(A, A, A, A, 64, 28672, 8192, 3, 128, 1, None) == 8          # 117 MB of partial sums: refused
    assert lib.potq_gemm_workspace_bytes(64, 13824, 5120, 3) <= 64 << 20  # the largest shape of config 5 fits
    assert lib.potq_gemm_workspace_bytes(16, 4096, 4096, 3) == 0          # up to 16 tokens: no workspace is used
    assert lib.potq_gemm_workspace_bytes(32, 4096, 4096, 3) == 16 * 32 * 4096 * 4
    assert lib.potq_gemm_workspace_bytes(256, 13824, 5120, 3) == 0      # enough output tiles: no split
    few_tiles = lib.potq_gemm_workspace_bytes(256, 4096, 4096, 3)         # too few output tiles: K is split
    assert few_tiles % (256 * 4096 * 4) == 0 and 2 <= few_tiles // (256 * 4096 * 4) <= 8
    assert lib.potq_gemm_workspace_bytes(0, 4096, 4096, 3) == 0
    assert lib.potq_gemm_workspace_bytes(32, 4096, 4100, 3) == 0          # shapes pot_gemm refuses need nothing
    assert lib.potq_gemm_workspace_bytes(32, 4096, 4096, 5) == 0 and lib.potq_gemm_workspace_bytes(32, 4100, 4096, 3) == 0
    # the exponent form of the GEMV: large 2- and 3-bit matrices with at least 32 groups per row
    assert lib.potq_gemv_exponent_form(28672, 8192, 3) == 1 and lib.potq_gemv_exponent_form(8192, 28672, 2) == 1
    assert lib.potq_gemv_exponent_form(4096, 4096, 3) == 0        # too small for the conversion of x to pay
    assert lib.potq_gemv_exponent_form(28672, 8192, 4) == 0       # +-2^7 does not fit a signed byte
    assert lib.potq_gemv_exponent_form(1 << 20, 2048, 3) == 0     # fewer than 32 groups per row
    assert lib.potq_gemv_exponent_form(0, 8192, 3) == 0 and lib.potq_gemv_exponent_form(28672, 8200, 3) == 0
    assert lib.potq_gemv_exponent_form(11008, 4096, 3) == 1       # rows for 160 workgroups: it pays from 24 M weights
    assert lib.potq_gemv_exponent_form(4096, 11008, 3) == 0       # too few rows
    # matrices sharing x: every size the form can serve
    lib.potq_gemv_batch_exponent_form.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int]
    assert lib.potq_gemv_batch_exponent_form(3, 4096, 3) == 1 and lib.potq_gemv_batch_exponent_form(2, 32768, 2) == 1
    assert lib.potq_gemv_batch_exponent_form(3, 2048, 3) == 0 and lib.potq_gemv_batch_exponent_form(3, 36864, 3) == 0
    assert lib.potq_gemv_batch_exponent_form(3, 4096, 4) == 0 and lib.potq_gemv_batch_exponent_form(17, 4096, 3) == 0
    assert lib.potq_gemv_batch_exponent_form(0, 4096, 3) == 0
    assert lib.int_gemv(A, A, A, MIS, A, 16, 128, 3, 128, 1, None) == ALIGN
    r = lib.potq_repack
    assert r(A, A, 24, 128, 3, 1, None) == SHAPE
    assert r(A, A, 16, 128, 3, 5, None) == LAYOUT
    assert r(A, None, 16, 128, 3, 1, None) == NULL
    qz = lib.pot_quantize
    assert qz(None, A, A, 16, 128, 3, 128, None) == NULL
    assert qz(A, A, A, 16, 128, 5, 128, None) == BITS
    assert qz(A, A, A, 16, 128, 3, 100, None) == GROUP
    assert qz(A, MIS, A, 16, 128, 3, 128, None) == ALIGN
    assert qz(None, None, None, 0, 128, 3, 128, None) == OK
    ff, fb = lib.pot_fakequant_forward, lib.pot_fakequant_backward
    assert ff(A, A, None, A, 16, 128, 3, 128, None) == NULL
    assert ff(A, A, A, A, 16, 128, 5, 128, None) == BITS
    assert ff(A, A, A, MIS, 16, 128, 3, 128, None) == ALIGN
    assert ff(None, None, None, None, 0, 128, 3, 128, None) == OK
    assert fb(A, A, A, None, A, 16, 128, 3, 128, None) == NULL
    assert fb(A, A, A, A, A, 16, 128, 3, 96, None) == GROUP
    assert fb(A, A, A, A, 0x10002, 16, 128, 3, 128, None) == ALIGN
    assert fb(None, None, None, None, None, 16, 0, 3, 128, None) == OK
    c = lib.pot_check_scales
    assert c(A, 4, 3, None, None) == NULL
    assert c(A, 4, 5, A, None) == BITS
    assert c(A, -1, 3, A, None) == SHAPE


def test_driver_entry_points_exist():
    import importlib
    entry = importlib.import_module("__graft_entry__")
    assert callable(entry.build) and callable(entry.smoke)


def test_build_step_loads_without_the_built_library():
    """build() must work in a tree that has no libpotq.so yet: it may not import the package, which needs it."""
    import subprocess
    import sys
    code = ("import sys, __graft_entry__ as g; m = g._build_module(); "
            "assert m.LIB_PATH.endswith('libpotq.so') and callable(m.build); "
            "assert not any(k.startswith('paper_2507_11959_amd') for k in sys.modules)")
    subprocess.run([sys.executable, "-c", code], check=True, cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def test_binding_rejects_mismatched_shapes_before_any_launch():
    """A wrong group size or a short scale / output tensor is a ValueError in the binding, never an
    out-of-bounds access on the device (host tensors suffice: the checks come before any pointer is taken)."""
    import torch
    from paper_2507_11959_amd import binding
    N, K, bits = 16, 256, 3
    codes = torch.zeros((N, K * bits // 8), dtype=torch.uint8)
    scales128 = torch.zeros((N, K // 128), dtype=torch.float16)
    x = torch.zeros((K,), dtype=torch.float16)
    with pytest.raises(ValueError, match="scales"):
        binding.pot_dequant(codes, scales128, K, bits, group=64)
    with pytest.raises(ValueError, match="out"):
        binding.pot_dequant(codes, scales128, K, bits, out=torch.zeros((N, K // 2), dtype=torch.float16))
    with pytest.raises(ValueError, match="zeros"):
        binding.int_dequant(codes, scales128, scales128[:, :1], K, bits)
    with pytest.raises(ValueError, match="scales"):
        binding.pot_gemv(codes, scales128[:8], x, K, bits)
    with pytest.raises(ValueError, match="y"):
        binding.pot_gemv(codes, scales128, x, K, bits, out=torch.zeros((N // 2,), dtype=torch.float16))
    with pytest.raises(ValueError, match="scales"):
        binding.pot_gemm(codes, scales128, x[None, :], K, bits, group=64)
    with pytest.raises(ValueError, match="Y"):
        binding.pot_gemm(codes, scales128, x[None, :], K, bits, out=torch.zeros((1, N + 16), dtype=torch.float16))
    with pytest.raises(ValueError, match="scales"):
        binding.make_batch([(codes, scales128, None, torch.zeros((N, K), dtype=torch.float16), K, bits)], group=64)
    with pytest.raises(ValueError, match="group"):
        binding.pot_dequant(codes, scales128, K, bits, group=32)
