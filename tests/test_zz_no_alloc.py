"""pot_gemm_noalloc (split-K partial sums in the library's built-in buffer) against pot_gemm
with a caller-supplied workspace, through the C ABI: same result bit for bit, on calls in a
row that share the buffer, the later ones with smaller inputs; plus the oracle on sampled rows."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import REL_TOL, dev, host_bits, rel_err

pytestmark = pytest.mark.gpu

# (M, N, K): 17..64 tokens split K over workgroups through the scratch buffer (checked below
# through the size query); the second call is smaller in every dimension, the third has more
# than 64 tokens on a matrix with few output tiles (the other kernel configuration that splits)
CALLS = [(64, 2048, 4096), (24, 512, 2048), (200, 1024, 2048)]


@pytest.mark.parametrize("bits", [3, 2])
def test_noalloc_equals_pot_gemm_on_calls_in_a_row(bits):
    from paper_2507_11959_amd import binding
    lib = binding.raw()
    G = 128
    stream = torch.cuda.current_stream().cuda_stream
    prepared = []
    for i, (M, N, K) in enumerate(CALLS):
        need = lib.potq_gemm_workspace_bytes(M, N, K, bits)
        assert 2 * M * N * 4 <= need <= 64 << 20, "the case must use the scratch buffer and fit it"
        packed = workloads.packed_codes(900 + 10 * i + bits, N, K, bits)
        scales = workloads.pot_scales(901 + 10 * i + bits, N, K, G)
        X = workloads.activations(902 + 10 * i + bits, M, K)
        tiled = binding.potq_repack(dev(packed), K, bits)
        ws = torch.empty((need,), dtype=torch.uint8, device="cuda:0")
        prepared.append((M, N, K, packed, scales, X, tiled, dev(scales), dev(X), ws,
                         torch.full((M, N), 3.0, dtype=torch.float16, device="cuda:0"),
                         torch.full((M, N), 5.0, dtype=torch.float16, device="cuda:0")))
    torch.cuda.synchronize()
    # every allocation is done: the calls under test, back to back on one stream
    for (M, N, K, packed, scales, X, tiled, d_s, d_X, ws, want, got) in prepared:
        assert lib.pot_gemm(tiled.data_ptr(), d_s.data_ptr(), d_X.data_ptr(), want.data_ptr(), M, N, K, bits, G,
                            binding.LAYOUT_TILE16, ws.data_ptr(), ws.numel(), stream) == 0
    for (M, N, K, packed, scales, X, tiled, d_s, d_X, ws, want, got) in prepared:
        assert lib.pot_gemm_noalloc(tiled.data_ptr(), d_s.data_ptr(), d_X.data_ptr(), got.data_ptr(), M, N, K, bits,
                                    G, binding.LAYOUT_TILE16, stream) == 0
    torch.cuda.synchronize()
    for (M, N, K, packed, scales, X, tiled, d_s, d_X, ws, want, got) in prepared:
        assert np.array_equal(host_bits(got), host_bits(want)), (M, N, K)
        rows = np.unique(np.concatenate([[0, 15, 16, N - 1], np.arange(7, N, 97)]))
        ref = oracle.gemm(packed[rows], scales[rows], None, X, K, bits, G)
        err, _, _ = rel_err(host_bits(got)[:, rows], ref, K)
        assert err <= REL_TOL, (M, N, K, err)


def test_noalloc_refuses_what_does_not_fit():
    from paper_2507_11959_amd import binding
    lib = binding.raw()
    M, N, K, bits = 64, 28672, 8192, 3
    assert lib.potq_gemm_workspace_bytes(M, N, K, bits) > 64 << 20
    t = torch.zeros((4096,), dtype=torch.uint8, device="cuda:0")
    p = t.data_ptr()        # never dereferenced: the call is refused on the host
    assert lib.pot_gemm_noalloc(p, p, p, p, M, N, K, bits, 128, binding.LAYOUT_TILE16, None) == 8
