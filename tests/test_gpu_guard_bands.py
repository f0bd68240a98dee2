"""Every entry point that writes device memory, run on outputs that sit between guard bands: the bytes
on either side of the output must be untouched afterwards (and the output itself fully written).  Shapes
are ragged on purpose: partial workgroups, tile sets that do not divide the grid, every GEMM configuration
class, the exponent form, the batch launches."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import DEV, Guarded, dev

pytestmark = pytest.mark.gpu
SENTINEL = 7.0      # a value none of the kernels can produce from these inputs everywhere at once


@pytest.fixture(scope="module")
def potq():
    import paper_2507_11959_amd as p
    return p


def _written(g: Guarded) -> bool:
    return not bool((g.tensor == SENTINEL).all())


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", [(1, 128), (37, 640), (129, 4096), (3083, 1152)])
def test_dequant_stays_inside_its_output(potq, bits, N, K):
    packed = dev(workloads.packed_codes(5 + bits, N, K, bits))
    S, Z = workloads.int_scales_zeros(6 + bits, N, K, bits, 128)
    for is_int in (False, True):
        g = Guarded((N, K), torch.float16, SENTINEL)
        if is_int:
            potq.int_dequant(packed, dev(S), dev(Z), K, bits, 128, out=g.tensor)
        else:
            potq.pot_dequant(packed, dev(workloads.pot_scales(7, N, K, 128)), K, bits, 128, out=g.tensor)
        torch.cuda.synchronize()
        assert g.intact() and _written(g), (bits, N, K, is_int)


@pytest.mark.parametrize("bits", [2, 3])
def test_dequant_batch_stays_inside_every_output(potq, bits):
    shapes = [(37, 640), (1, 128), (16, 2048), (129, 4096), (5, 11008), (3083, 1152)]
    guards, mats = [], []
    for i, (N, K) in enumerate(shapes):
        g = Guarded((N, K), torch.float16, SENTINEL)
        guards.append(g)
        mats.append((dev(workloads.packed_codes(40 + i, N, K, bits)), dev(workloads.pot_scales(50 + i, N, K, 128)),
                     g.tensor, K))
    potq.pot_dequant_batch(mats, bits, 128)
    torch.cuda.synchronize()
    for g, shape in zip(guards, shapes):
        assert g.intact() and _written(g), shape


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_repack_and_quantize_stay_inside_their_outputs(potq, bits):
    N, K = 48, 1152
    packed = dev(workloads.packed_codes(60 + bits, N, K, bits))
    g = Guarded(tuple(packed.shape), torch.uint8)
    potq.potq_repack(packed, K, bits, out=g.tensor)
    torch.cuda.synchronize()
    assert g.intact()
    from paper_2507_11959_amd import binding
    W = dev(workloads.weights_f16(61 + bits, N, K))
    gc, gs = Guarded((N, K * bits // 8), torch.uint8), Guarded((N, K // 128), torch.float16)
    assert binding.raw().pot_quantize(W.data_ptr(), gc.tensor.data_ptr(), gs.tensor.data_ptr(), N, K, bits, 128,
                                      torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    assert gc.intact() and gs.intact()
    gamma = torch.zeros((N, K // 128), dtype=torch.float32, device=DEV)
    gq, gd = Guarded((N, K), torch.float16, SENTINEL), Guarded((N, K // 128), torch.float32)
    lib = binding.raw()
    st = torch.cuda.current_stream().cuda_stream
    assert lib.pot_fakequant_forward(W.data_ptr(), gs.tensor.data_ptr(), gamma.data_ptr(), gq.tensor.data_ptr(), N, K,
                                     bits, 128, st) == 0
    assert lib.pot_fakequant_backward(W.data_ptr(), gs.tensor.data_ptr(), gamma.data_ptr(), W.data_ptr(),
                                      gd.tensor.data_ptr(), N, K, bits, 128, st) == 0
    torch.cuda.synchronize()
    assert gq.intact() and gd.intact() and _written(gq)


@pytest.mark.parametrize("N,K,bits", [(16, 128, 3), (48, 1152, 2), (4112, 4096, 3), (1040, 16384, 4),
                                      (8208, 8192, 3),       # exponent form, 513 row tiles
                                      (15904, 4224, 2)])     # exponent form, ragged group count
def test_gemv_stays_inside_its_output(potq, N, K, bits):
    tiled = potq.potq_repack(dev(workloads.packed_codes(70 + bits, N, K, bits)), K, bits)
    x = dev(workloads.activations(71, 1, K)[0])
    S, Z = workloads.int_scales_zeros(72 + bits, N, K, bits, 128)
    for is_int in (False, True):
        g = Guarded((N,), torch.float16, SENTINEL)
        if is_int:
            potq.int_gemv(tiled, dev(S), dev(Z), x, K, bits, out=g.tensor)
        else:
            potq.pot_gemv(tiled, dev(workloads.pot_scales(73, N, K, 128)), x, K, bits, out=g.tensor)
        torch.cuda.synchronize()
        assert g.intact() and _written(g), (N, K, bits, is_int)


@pytest.mark.parametrize("bits", [2, 3])
def test_gemv_batch_stays_inside_every_output(potq, bits):
    from paper_2507_11959_amd import binding
    K = 4096
    for rows in ((48, 16, 1040), (11008, 5504, 16)):           # fp16 form, exponent form
        x = dev(workloads.activations(80, 1, K)[0])
        guards, items = [], []
        for i, N in enumerate(rows):
            g = Guarded((N,), torch.float16, SENTINEL)
            guards.append(g)
            items.append((potq.potq_repack(dev(workloads.packed_codes(81 + i, N, K, bits)), K, bits),
                          dev(workloads.pot_scales(82 + i, N, K, 128)), None, g.tensor))
        arr = binding.make_gemv_batch(items, K, bits)
        assert binding.raw().pot_gemv_batch(arr, len(items), x.data_ptr(), K, bits, 128, binding.LAYOUT_TILE16,
                                            torch.cuda.current_stream().cuda_stream) == 0
        torch.cuda.synchronize()
        for g in guards:
            assert g.intact() and _written(g), rows


@pytest.mark.parametrize("M,N,K", [(2, 1040, 1152), (3, 16400, 8192),      # multi-vector GEMV forms
                                   (7, 48, 1152), (16, 1040, 2048),        # few-token kernel
                                   (17, 1040, 2048), (40, 2064, 4096), (64, 8192, 8192),
                                   (24, 272, 9216),                        # split over workgroups (workspace)
                                   (100, 1040, 2048), (200, 4112, 1152), (300, 528, 2048)])
def test_gemm_stays_inside_its_output_and_workspace(potq, M, N, K):
    bits = 3
    tiled = potq.potq_repack(dev(workloads.packed_codes(90, N, K, bits)), K, bits)
    S = dev(workloads.pot_scales(91, N, K, 128))
    X = dev(workloads.activations(92, M, K))
    from paper_2507_11959_amd import binding
    need = binding.raw().potq_gemm_workspace_bytes(M, N, K, bits)
    ws = Guarded((max(need, 16),), torch.uint8)
    g = Guarded((M, N), torch.float16, SENTINEL)
    potq.pot_gemm(tiled, S, X, K, bits, out=g.tensor, workspace=ws.tensor if need else None)
    torch.cuda.synchronize()
    assert g.intact() and ws.intact() and _written(g), (M, N, K)
    g2 = Guarded((M, N), torch.float16, SENTINEL)
    potq.pot_gemm_noalloc(tiled, S, X, g2.tensor, K, bits)
    torch.cuda.synchronize()
    assert g2.intact() and torch.equal(g.tensor, g2.tensor), (M, N, K)


def test_check_scales_writes_one_word(potq):
    from paper_2507_11959_amd import binding
    s = dev(workloads.pot_scales(99, 33, 1152, 128))
    g = Guarded((1,), torch.int64)
    assert binding.raw().pot_check_scales(s.data_ptr(), s.numel(), 3, g.tensor.data_ptr(),
                                          torch.cuda.current_stream().cuda_stream) == 0
    torch.cuda.synchronize()
    assert g.intact() and int(g.tensor.item()) == 0
