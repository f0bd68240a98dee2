"""Pins for the oracle's software binary16 conversions: numpy's float16 is the
outside authority (a library type the oracle does not use)."""
import numpy as np

import oracle


def test_half_to_double_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], ref[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


def test_double_to_half_roundtrip_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    vals = bits.view(np.float16).astype(np.float64)
    for b, v in zip(bits, vals):
        if np.isnan(v):
            continue
        assert oracle.double_to_half(float(v)) == int(b)


def test_double_to_half_midpoints_and_neighbours():
    # every midpoint between adjacent non-negative finite fp16 values, and a nudge either side
    pos = np.arange(0, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    nxt = np.append(pos[1:], 65536.0)       # the value after 65504 would be 2^16
    mid = 0.5 * (pos + nxt)
    cases = np.concatenate([mid, np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf)])
    cases = np.concatenate([cases, -cases])
    with np.errstate(over="ignore"):
        ref = cases.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half(float(c)) for c in cases], dtype=np.uint16)
    assert np.array_equal(got, ref)


def test_double_to_half_random_and_specials():
    rng = np.random.default_rng(7)
    x = np.concatenate([
        rng.standard_normal(20000),
        rng.standard_normal(20000) * 1e-6,
        rng.standard_normal(20000) * 3e4,
        np.exp(rng.uniform(-20, 12, 20000)) * rng.choice([-1.0, 1.0], 20000),
        [0.0, -0.0, np.inf, -np.inf, 65504.0, 65519.999, 65520.0, 2.0 ** -24, 2.0 ** -25,
         np.nextafter(2.0 ** -25, 1.0), 1e300, -1e300, 5e-324],
    ])
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, ref)
    assert oracle.double_to_half(float("nan")) & 0x7C00 == 0x7C00
    assert oracle.double_to_half(float("nan")) & 0x03FF != 0
