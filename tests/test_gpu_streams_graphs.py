"""The entry points only enqueue work on the caller's stream: they must work on a
non-default stream and inside HIP graph capture (no allocation, no synchronisation,
no memset nodes), and a captured graph must give the eager results on every replay."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import dev, host_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def potq():
    import paper_2507_11959_amd as p
    return p


def _layer(potq, bits, K=1024):
    G = 128
    mats = []
    for i, N in enumerate([64, 48, 160]):
        packed, scales = workloads.pot_matrix(9, i, N, K, bits, G)
        mats.append(dict(N=N, packed=packed, scales=scales, codes=dev(packed), s=dev(scales),
                         tiled=potq.potq_repack(dev(packed), K, bits),
                         out=torch.empty((N, K), dtype=torch.float16, device="cuda:0")))
    return mats


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_non_default_stream(potq, bits):
    K = 1024
    mats = _layer(potq, bits, K)
    x = dev(workloads.activations(5, 1, K)[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        potq.pot_dequant_batch([(m["codes"], m["s"], m["out"], K) for m in mats], bits)
        ys = potq.pot_gemv_batch([(m["tiled"], m["s"]) for m in mats], x, K, bits)
    side.synchronize()
    for m, y in zip(mats, ys):
        assert np.array_equal(host_bits(m["out"]), oracle.pot_dequant(m["packed"], m["scales"], K, bits, 128))
        assert torch.equal(y, potq.pot_gemv(m["tiled"], m["s"], x, K, bits))


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_graph_capture_and_replay(potq, bits):
    K, M = 1024, 24
    mats = _layer(potq, bits, K)
    x = dev(workloads.activations(6, 1, K)[0])
    X = dev(workloads.activations(7, M, K))
    m0 = mats[0]
    ws = potq.gemm_workspace(M, m0["N"], K, bits)
    y_g = [torch.empty((m["N"],), dtype=torch.float16, device="cuda:0") for m in mats]
    Y_g = torch.empty((M, m0["N"]), dtype=torch.float16, device="cuda:0")
    from paper_2507_11959_amd import binding
    batch = binding.make_gemv_batch([(m["tiled"], m["s"], None, y) for m, y in zip(mats, y_g)], K, bits)
    lib = binding.raw()

    # eager reference results
    eager_y = [potq.pot_gemv(m["tiled"], m["s"], x, K, bits) for m in mats]
    eager_Y = potq.pot_gemm(m0["tiled"], m0["s"], X, K, bits, workspace=ws)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        st = torch.cuda.current_stream().cuda_stream
        potq.pot_dequant_batch([(m["codes"], m["s"], m["out"], K) for m in mats], bits)
        assert lib.pot_gemv_batch(batch, len(mats), x.data_ptr(), K, bits, 128, 1, st) == 0
        potq.pot_gemm(m0["tiled"], m0["s"], X, K, bits, out=Y_g, workspace=ws)
    for replay in range(3):
        for m in mats:
            m["out"].zero_()                 # the program's own eager work between replays
        for y in y_g:
            y.zero_()
        Y_g.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for m, y, ey in zip(mats, y_g, eager_y):
            assert np.array_equal(host_bits(m["out"]), oracle.pot_dequant(m["packed"], m["scales"], K, bits, 128))
            assert torch.equal(y, ey), replay
        assert torch.equal(Y_g, eager_Y), replay


def test_graph_capture_of_the_exponent_form_with_long_rows(potq):
    """The 16-wavefront exponent-form GEMV needs more LDS than a kernel's default limit; raising
    the limit is not stream work and must not disturb a capture."""
    N, K, bits = 4112, 16384, 3
    assert potq.potq_gemv_exponent_form(N, K, bits)
    packed, scales = workloads.pot_matrix(9, 40, N, K, bits, 128)
    tiled, s = potq.potq_repack(dev(packed), K, bits), dev(scales)
    x = dev(workloads.activations(8, 1, K)[0])
    y_g = torch.empty((N,), dtype=torch.float16, device="cuda:0")
    from paper_2507_11959_amd import binding
    lib = binding.raw()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        st = torch.cuda.current_stream().cuda_stream
        assert lib.pot_gemv(tiled.data_ptr(), s.data_ptr(), x.data_ptr(), y_g.data_ptr(), N, K, bits, 128, 1, st) == 0
    eager = potq.pot_gemv(tiled, s, x, K, bits)
    for replay in range(3):
        y_g.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y_g, eager), replay
