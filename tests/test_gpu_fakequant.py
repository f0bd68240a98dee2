"""GPU parity of the Step 2 op (Sec. 3.3): forward bit-exact, backward within fp32 summation error."""
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


def _inputs(seed, N, K, bits, group, gamma_span=0.3):
    rng = np.random.default_rng(seed)
    W = workloads.weights_f16(seed, N, K)
    if N:
        W[0, :7] = [0.0, -0.0, 6e-8, -6e-8, 65504.0, -65504.0, 1.0]          # zeros, subnormals, the largest fp16
    _, S = oracle.pot_quantize(W, bits, group, nthreads=8)
    Gamma = rng.uniform(-gamma_span, gamma_span, size=S.shape).astype(np.float32)
    dWq = (rng.standard_normal((N, K)) * 1e-2).astype(np.float16)
    return W, S.view(np.float16), Gamma, dWq


def _check(potq, W, S, Gamma, dWq, bits, group):
    N, K = W.shape
    got_f = host_bits(potq.pot_fakequant_forward(dev(W), dev(S), torch.from_numpy(Gamma).cuda(), bits, group))
    want_f = oracle.fakequant_forward(W, S, Gamma, bits, group, nthreads=8)
    assert np.array_equal(got_f, want_f)
    got_b = potq.pot_fakequant_backward(dev(W), dev(S), torch.from_numpy(Gamma).cuda(), dev(dWq), bits,
                                        group).cpu().numpy()
    want_b = oracle.fakequant_backward(W, S, Gamma, dWq, bits, group, nthreads=8)
    # fp32 sum of `group` exact products in a fixed tree order against the binary64 sum:
    # |error| <= (log2(group) + 8) * 2^-24 * S * sum |terms|; the bound uses 2^qmax * |dWq| for the terms
    qmax = 2 ** (bits - 1) - 1
    bound = 16 * 2.0 ** -24 * S.astype(np.float64) * \
        (np.abs(dWq.astype(np.float64)) * 2.0 ** qmax).reshape(N, K // group, group).sum(axis=2)
    assert np.all(np.abs(got_b.astype(np.float64) - want_b.astype(np.float64)) <= bound + 1e-30)
    return got_b, want_b


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("N,K", [(1, 128), (7, 640), (33, 1024), (3, 11008)])
def test_fakequant_vs_oracle(potq, bits, group, N, K):
    W, S, Gamma, dWq = _inputs(31 * N + K + bits + group, N, K, bits, group)
    got_b, want_b = _check(potq, W, S, Gamma, dWq, bits, group)
    assert np.abs(want_b).max() > 0


@pytest.mark.parametrize("bits", [2, 3])
def test_fakequant_gamma_zero_and_extremes(potq, bits):
    N, K, group = 16, 512, 128
    W, S, Gamma, dWq = _inputs(900 + bits, N, K, bits, group)
    Gamma[:] = 0
    _check(potq, W, S, Gamma, dWq, bits, group)
    Gamma[:] = np.float32(-0.999)           # nearly vanishing scale: every weight above range
    _check(potq, W, S, Gamma, dWq, bits, group)
    Gamma[:] = np.float32(1000.0)           # huge scale: every weight below range
    _check(potq, W, S, Gamma, dWq, bits, group)
    Gamma[:] = np.float32(-1.5)             # outside the method (S^ < 0): still the same as the oracle
    _check(potq, W, S, Gamma, dWq, bits, group)


def test_fakequant_full_size_layer_matrix(potq):
    # one Llama-2-7B MLP matrix (11008 x 4096), 3-bit, as in the launch configuration the benchmark times
    bits, group, N, K = 3, 128, 11008, 4096
    W, S, Gamma, dWq = _inputs(4242, N, K, bits, group, gamma_span=0.05)
    _check(potq, W, S, Gamma, dWq, bits, group)


def test_fakequant_empty(potq):
    W = torch.empty((0, 256), dtype=torch.float16, device="cuda:0")
    S = torch.empty((0, 2), dtype=torch.float16, device="cuda:0")
    G = torch.empty((0, 2), dtype=torch.float32, device="cuda:0")
    assert potq.pot_fakequant_forward(W, S, G, 3).shape == (0, 256)
    assert potq.pot_fakequant_backward(W, S, G, W, 3).shape == (0, 2)
