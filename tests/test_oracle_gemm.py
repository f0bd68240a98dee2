"""Pins for the oracle's GEMV / GEMM: special cases with exact answers and
numpy's float64 matmul of the independently de-quantised matrix."""
import numpy as np
import pytest

import oracle
import np_reference as ref
import workloads


def _f16(bits_arr):
    return np.asarray(bits_arr, dtype=np.uint16).view(np.float16)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_gemv_one_hot_returns_columns_exactly(bits):
    N, K, G = 20, 384, 128
    packed, scales = workloads.pot_matrix(2, 0, N, K, bits, G)
    W = oracle.pot_dequant(packed, scales, K, bits, G)
    for k in (0, 1, 127, 128, 200, K - 1):
        x = np.zeros(K, dtype=np.float16)
        x[k] = 1.0
        y = oracle.gemv(packed, scales, None, x, K, bits, G)
        assert np.array_equal(y, W[:, k])


def test_gemv_all_ones_zero_codes_is_group_sum_of_scales():
    N, K, G = 16, 512, 128
    scales = (2.0 ** -np.arange(4)[None, :] * np.ones((N, 1))).astype(np.float16)   # exactly summable
    packed = np.zeros((N, K * 3 // 8), dtype=np.uint8)
    y = oracle.gemv(packed, scales, None, np.ones(K, np.float16), K, 3, G)
    assert np.all(_f16(y).astype(np.float64) == G * scales.astype(np.float64).sum(axis=1))


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_gemv_sign_flip_negates(bits):
    N, K, G = 12, 256, 128
    packed, scales = workloads.pot_matrix(2, 1, N, K, bits, G)
    codes = oracle.unpack_codes(packed, K, bits)
    flipped = oracle.pack_codes(codes ^ np.uint8(1 << (bits - 1)), bits)
    x = workloads.activations(5, 1, K)[0]
    y0, f0 = oracle.gemv(packed, scales, None, x, K, bits, G, want_f64=True)
    y1, f1 = oracle.gemv(flipped, scales, None, x, K, bits, G, want_f64=True)
    assert np.array_equal(f0, -f1)
    assert np.array_equal(y0 ^ 0x8000, y1)


@pytest.mark.parametrize("bits,M", [(2, 1), (3, 1), (3, 5)])
def test_gemm_vs_numpy_float64_matmul(bits, M):
    N, K, G = 32, 640, 128
    packed, scales = workloads.pot_matrix(4, 0, N, K, bits, G)
    X = workloads.activations(workloads.seed_of(4, 0, 2), M, K)
    Y, Y64 = oracle.gemm(packed, scales, None, X, K, bits, G, want_f64=True)
    W = ref.pot_dequant(packed, scales, K, bits, G)
    want = ref.gemm_f64(W, X)
    assert Y64.shape == (M, N)
    assert np.allclose(Y64, want, rtol=1e-12, atol=1e-13)
    # the fp16 result is the single rounding of the sum (allow numpy's different summation order
    # to flip a rounding only where the sum sits within 1e-12 of a midpoint: none do here)
    assert np.array_equal(Y, want.astype(np.float16).view(np.uint16))
    # every row of a GEMM is the GEMV of that row; threads do not matter
    for m in range(M):
        assert np.array_equal(oracle.gemv(packed, scales, None, X[m], K, bits, G), Y[m])
    assert np.array_equal(oracle.gemm(packed, scales, None, X, K, bits, G, nthreads=3), Y)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_int_gemm_vs_numpy(bits):
    N, K, G, M = 24, 512, 128, 3
    packed, S, Z = workloads.int_matrix(4, 1, N, K, bits, G)
    X = workloads.activations(9, M, K)
    Y, Y64 = oracle.gemm(packed, S, Z, X, K, bits, G, want_f64=True)
    W = ref.int_dequant(packed, S, Z, K, bits, G)
    want = ref.gemm_f64(W, X)
    assert np.allclose(Y64, want, rtol=1e-12, atol=1e-13)
    assert np.array_equal(Y, want.astype(np.float16).view(np.uint16))
    # one-hot rows give exact columns of the de-quantised matrix
    E = np.zeros((2, K), np.float16)
    E[0, 3] = 1.0
    E[1, 300] = 1.0
    Yc = oracle.gemm(packed, S, Z, E, K, bits, G)
    Wd = oracle.int_dequant(packed, S, Z, K, bits, G)
    assert np.array_equal(Yc[0], Wd[:, 3]) and np.array_equal(Yc[1], Wd[:, 300])


def test_transposed_group_reading_is_caught():
    # scales vary along K only: if groups ran along N instead, this would fail
    N, K, G = 256, 256, 128
    scales = np.tile(np.array([[0.5, 0.25]], np.float16), (N, 1))
    packed = np.zeros((N, K * 2 // 8), np.uint8)
    W = _f16(oracle.pot_dequant(packed, scales, K, 2, G)).astype(np.float64)
    assert np.all(W[:, :128] == 0.5) and np.all(W[:, 128:] == 0.25)
