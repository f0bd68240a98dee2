"""GPU parity of pot_gemv / int_gemv on the canonical layout (the boundary's own format, consumed without
potq_repack): one-hot activations give exact columns of the de-quantised matrix, random activations sit
inside the gate, row counts need not be multiples of 16, both group sizes, rows beyond 64 KB of LDS, and a
70B-sized matrix on sampled rows.  The tiled path on the same inputs must agree with it to the same gate."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import REL_TOL, Guarded, dev, host_bits, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def potq():
    import paper_2507_11959_amd as p
    return p


def _inputs(seed, N, K, bits, group, is_int):
    packed = workloads.packed_codes(seed, N, K, bits)
    if is_int:
        S, Z = workloads.int_scales_zeros(seed + 1, N, K, bits, group)
    else:
        S, Z = workloads.pot_scales(seed + 1, N, K, group), None
    return packed, S, Z


def _gemv(potq, packed, S, Z, x, K, bits, group, out=None):
    if Z is None:
        return potq.pot_gemv(dev(packed), dev(S), dev(x), K, bits, group, layout=potq.LAYOUT_CANONICAL, out=out)
    return potq.int_gemv(dev(packed), dev(S), dev(Z), dev(x), K, bits, group, layout=potq.LAYOUT_CANONICAL, out=out)


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K,group", [(1, 128, 128), (37, 640, 64), (129, 4096, 128), (5, 11008, 128)])
def test_one_hot_gives_exact_columns(potq, bits, N, K, group, is_int):
    packed, S, Z = _inputs(400 + N + bits, N, K, bits, group, is_int)
    W = oracle.int_dequant(packed, S, Z, K, bits, group) if is_int else oracle.pot_dequant(packed, S, K, bits, group)
    rng = np.random.default_rng(N + K)
    for k in sorted(set([0, 1, 7, 8, 63, 64, 127, K - 128, K - 1] + list(rng.integers(0, K, 16)))):
        x = np.zeros((K,), np.float16)
        x[k] = 1.0
        assert np.array_equal(host_bits(_gemv(potq, packed, S, Z, x, K, bits, group)), W[:, k]), k


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K,group", [(1, 128, 128), (37, 640, 64), (273, 4096, 128), (70, 11008, 64),
                                       (1000, 8192, 128), (9001, 1152, 128)])
def test_vs_oracle_and_guard_bands(potq, bits, N, K, group, is_int):
    packed, S, Z = _inputs(500 + N + bits, N, K, bits, group, is_int)
    x = workloads.activations(501 + K, 1, K)
    want = oracle.gemm(packed, S, Z, x, K, bits, group, nthreads=8)[0]
    g = Guarded((N,), torch.float16, 7.0)
    _gemv(potq, packed, S, Z, x[0], K, bits, group, out=g.tensor)
    torch.cuda.synchronize()
    assert g.intact()
    e, nw, nfloor = rel_err(host_bits(g.tensor), want, K)
    assert e <= REL_TOL, (e, nw, nfloor)


@pytest.mark.parametrize("K", [32768, 81920])
def test_rows_beyond_64_kib_of_lds(potq, K):
    N, bits = 48, 3
    packed, S, Z = _inputs(600 + K, N, K, bits, 128, False)
    x = workloads.activations(601 + K, 1, K)
    want = oracle.gemm(packed, S, None, x, K, bits, 128, nthreads=8)[0]
    e, nw, nfloor = rel_err(host_bits(_gemv(potq, packed, S, None, x[0], K, bits, 128)), want, K)
    assert e <= REL_TOL, (e, nw, nfloor)
    from paper_2507_11959_amd import binding
    t = torch.zeros((4096,), dtype=torch.uint8, device="cuda:0")
    assert binding.raw().pot_gemv(t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(), 16, 81920 + 128, bits, 128,
                                  binding.LAYOUT_CANONICAL, None) == 4


@pytest.mark.parametrize("bits", [2, 3])
def test_70b_sized_matrix_sampled_rows_and_the_tiled_path(potq, bits):
    N, K = 28672, 8192
    rng = np.random.default_rng(bits)
    packed, S = workloads.pot_matrix(3, 4, N, K, bits, 128)
    x = workloads.activations(workloads.seed_of(3, 4, 2), 1, K)
    y_c = potq.pot_gemv(dev(packed), dev(S), dev(x[0]), K, bits, layout=potq.LAYOUT_CANONICAL)
    y_t = potq.pot_gemv(potq.potq_repack(dev(packed), K, bits), dev(S), dev(x[0]), K, bits)
    rows = np.unique(np.concatenate([[0, 1, 7, 8, N - 9, N - 1], rng.integers(0, N, 1500)]))
    want = oracle.gemm(packed[rows], S[rows], None, x, K, bits, 128, nthreads=8)[0]
    idx = torch.from_numpy(rows).to("cuda:0")
    for y in (y_c, y_t):
        e, nw, nfloor = rel_err(host_bits(y[idx]), want, K)
        assert e <= REL_TOL, (e, nw, nfloor)
    assert bool(torch.isfinite(y_c).all())


def test_non_finite_activations_follow_the_definition(potq):
    N, K, bits = 64, 1152, 3
    packed, S, Z = _inputs(700, N, K, bits, 128, False)
    x = workloads.activations(701, 1, K)[0]
    x[5], x[700] = np.float16(np.inf), np.float16(np.inf)
    want = oracle.gemm(packed, S, None, x[None, :], K, bits, 128)[0].view(np.float16)
    got = host_bits(_gemv(potq, packed, S, None, x, K, bits, 128)).view(np.float16)
    assert np.array_equal(np.isnan(got), np.isnan(want)) and np.array_equal(got[~np.isnan(want)], want[~np.isnan(want)])
