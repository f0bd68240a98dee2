"""GPU parity of pot_quantize (Step 1 scale search, Algorithm 1) against the CPU oracle:
integer decisions (codes, chosen multiplier via the scale) must agree bit for bit."""
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


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("N,K", [(1, 128), (7, 640), (24, 1024), (3, 11008)])
def test_quantize_bit_exact(potq, bits, group, N, K):
    W = workloads.weights_f16(900 + N + K + bits + group, N, K)
    W[0, : min(K, 130)] *= np.float16(40.0)            # a group with large weights
    if N > 2:
        W[1, :128] = 0                                  # an all-zero group
        W[2, 5] = np.float16(-0.5)                      # an outlier
    want_codes, want_scales = oracle.pot_quantize(W, bits, group, nthreads=8)
    codes, scales = potq.pot_quantize(dev(W), bits, group)
    assert np.array_equal(host_bits(scales), want_scales)
    assert np.array_equal(codes.cpu().numpy(), oracle.pack_codes(want_codes, bits))
    assert potq.pot_check_scales(scales, bits) == 0


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_quantize_then_dequant_round_trip(potq, bits):
    N, K, G = 256, 4096, 128
    W = workloads.weights_f16(77 + bits, N, K)
    codes, scales = potq.pot_quantize(dev(W), bits, G)
    Wd = potq.pot_dequant(codes, scales, K, bits, G)
    want_codes, want_scales = oracle.pot_quantize(W, bits, G, nthreads=8)
    want = oracle.pot_dequant(oracle.pack_codes(want_codes, bits), want_scales, K, bits, G, nthreads=8)
    assert np.array_equal(host_bits(Wd), want)
    # the reconstruction error is what PoT at this width can do on Gaussian weights (sanity, not parity)
    rel = float(((Wd.float().cpu() - torch.from_numpy(W).float()) ** 2).sum() / (torch.from_numpy(W).float() ** 2).sum())
    assert rel < (0.2 if bits == 3 else 0.45)


def test_quantize_empty(potq):
    from paper_2507_11959_amd import binding
    assert binding.raw().pot_quantize(None, None, None, 0, 128, 3, 128, None) == 0
