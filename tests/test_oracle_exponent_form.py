"""CPU pins for the exponent form of the fused GEMV (Sec. 4.2: a power-of-two weight only adds
to the exponent of the activation it meets, so the scale may be applied after the group's sum).

Checked here, without a GPU and in exact integer arithmetic:
  * inside the scale domain the oracle's de-quantised weights satisfy W~ = +-2^E * s exactly, so
    sum_g s_g * sum_{k in g} (+-2^E) x_k is the very sum the fused GEMV is defined by;
  * outside the domain it is not (the library's header says the two forms differ there);
  * the fixed-point representation the kernel uses for the activations of a scale group:
    k = 44 - max(largest exponent field of the group, 1) keeps |x * 2^k| below 2^30, is exact for
    every element within 2^19 of the group's largest one, and the signed base-256 digits obtained
    by adding 0x00808080 reproduce the integer."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
import workloads


def _exact(bits16: np.ndarray) -> list:
    """fp16 bit patterns -> exact rationals."""
    return [Fraction(float(v)) for v in bits16.view(np.float16).astype(np.float64).ravel()]


@pytest.mark.parametrize("bits", [2, 3])
@pytest.mark.parametrize("group", [64, 128])
def test_scale_leaves_the_inner_sum_inside_the_domain(bits, group):
    N, K = 4, 256
    packed, scales = workloads.pot_matrix(8, bits, N, K, bits, group)
    assert oracle.check_scales(scales, bits) == 0
    x = workloads.activations(8, 1, K)[0]
    W = oracle.pot_dequant(packed, scales, K, bits, group)
    codes = oracle.unpack_codes(packed, K, bits)
    xs = _exact(x.view(np.uint16))
    for n in range(N):
        w = _exact(W[n])
        direct = sum(wk * xk for wk, xk in zip(w, xs))
        s = _exact(scales[n])
        by_group = Fraction(0)
        for g in range(K // group):
            inner = Fraction(0)
            for k in range(g * group, (g + 1) * group):
                c = int(codes[n, k])
                sign, e = c >> (bits - 1), c & ((1 << (bits - 1)) - 1)
                inner += (-1 if sign else 1) * (1 << e) * xs[k]
            by_group += s[g] * inner
        assert by_group == direct


def test_outside_the_domain_the_two_forms_differ():
    # exponent field 30 and E = 3: the integer add wraps into the sign bit, the product overflows fp16
    bits, K = 3, 128
    codes = np.full((1, K), 3, dtype=np.uint8)              # +2^3 everywhere
    packed = oracle.pack_codes(codes, bits)
    scales = np.array([[0x7800]], dtype=np.uint16)          # 2^15, exponent field 30
    assert oracle.check_scales(scales, bits) == 1
    W = oracle.pot_dequant(packed, scales, K, bits, 128).view(np.float16).astype(np.float64)
    assert not np.allclose(W, 8.0 * 32768.0)


@pytest.mark.parametrize("seed", range(4))
def test_fixed_point_digits_of_the_activations(seed):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal(4096) * np.exp2(rng.integers(-22, 6, 4096))).astype(np.float16)
    x[7] = np.float16(65504.0) if seed == 0 else x[7]
    for g in range(0, 4096, 128):                           # every scale group against its own largest exponent
        _check_fixed_point_of_a_group(x[g:g + 128])
    _check_fixed_point_of_a_group(np.zeros(128, np.float16))             # exponent field 0 counts as 1
    _check_fixed_point_of_a_group(np.full(128, 6e-8, np.float16))        # subnormals only


def _check_fixed_point_of_a_group(x):
    bits16 = x.view(np.uint16)
    e = max(int((bits16 & 0x7FFF).max()) >> 10, 1)
    k = 44 - e
    largest = float(np.abs(x.astype(np.float64)).max())
    for v in x.astype(np.float64):
        scaled = Fraction(float(v)) * (1 << k)
        m = round(scaled)                                   # ties to even, as rintf does
        assert abs(m) < 2 ** 30
        if v != 0.0 and abs(v) * 2.0 ** 19 >= largest:
            assert scaled == m                              # exact within 2^19 of the largest element
        assert abs(scaled - m) <= Fraction(1, 2)            # else rounded to 2^-k <= 2^-29 * largest
        u = (m + 0x00808080) & 0xFFFFFFFF
        digits = [((u >> (8 * p)) & 0xFF) ^ (0x80 if p < 3 else 0) for p in range(4)]
        signed = [d - 256 if d >= 128 else d for d in digits]
        assert sum(d * 256 ** p for p, d in enumerate(signed)) == m
