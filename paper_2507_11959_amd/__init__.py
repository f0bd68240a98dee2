"""potq: MI355X-native power-of-two weight de-quantisation (PoT-PTQ, arXiv 2507.11959).

`csrc/` holds the gfx950 HIP kernels and the C ABI (declared in include/potq.h);
`binding` is the ctypes marshalling layer with the same entry-point names.
"""
from .binding import (  # noqa: F401
    LAYOUT_CANONICAL, LAYOUT_TILE16, PotqError, gemm_workspace, int_dequant, int_gemm, int_gemv, packed_bytes, packed_row_bytes,
    pot_check_scales, pot_quantize, pot_fakequant_forward, pot_fakequant_backward, pot_dequant, pot_dequant_batch, int_dequant_batch, pot_gemv_batch, int_gemv_batch, pot_gemm, pot_gemm_noalloc, pot_gemv, potq_gemv_exponent_form, potq_gemv_batch_exponent_form, potq_repack, strerror, version,
)
