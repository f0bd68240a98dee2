"""Pins for the decode: the paper's closed form (golden file written by hand),
exhaustive code x scale enumeration against numpy's float16 ldexp, and the
domain on which the Sec. 4.2 integer-add recipe equals the definition."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "pot_grid.txt")


def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            b, code, s, w = line.split()
            rows.append((int(b), int(code, 2), int(s, 16), int(w, 16)))
    return rows


def test_golden_grid_definition_and_recipe():
    rows = _golden_rows()
    assert len(rows) >= 30
    for bits, code, s, want in rows:
        assert oracle.decode_def(code, s, bits) == want, (bits, code, hex(s))
        assert oracle.decode_bits(code, s, bits) == want, (bits, code, hex(s))


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_grid_closed_form(bits):
    # Sec. 3.1: levels are s * {+-2^0 .. +-2^qmax}; all 2^b codes valid, distinct, non-zero
    qmax = 2 ** (bits - 1) - 1
    for s in (1.0, 0.0625, 0.0712890625, 3.0):
        sb = int(np.float16(s).view(np.uint16))
        vals = [oracle.half_to_double(oracle.decode_def(c, sb, bits)) for c in range(2 ** bits)]
        want = [float(np.float16(s)) * 2.0 ** e for e in range(qmax + 1)]
        want = want + [-v for v in want]          # sign bit is the MSB: codes >= 2^(b-1) are negative
        assert vals == want
        assert len(set(vals)) == 2 ** bits and 0.0 not in vals


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_exhaustive_codes_times_scales_vs_numpy(bits):
    qmax = 2 ** (bits - 1) - 1
    sbits = np.arange(65536, dtype=np.uint16)
    s16 = sbits.view(np.float16)
    lo, hi = 0x0400, (31 - qmax) << 10        # positive normal, exponent field 1 .. 30 - qmax
    in_dom = (sbits >= lo) & (sbits < hi)
    assert in_dom.sum() == (30 - qmax) * 1024
    for code in range(2 ** bits):
        sign, E = code >> (bits - 1), code & (2 ** (bits - 1) - 1)
        d = np.array([oracle.decode_def(code, int(b), bits) for b in sbits], dtype=np.uint16)
        r = np.array([oracle.decode_bits(code, int(b), bits) for b in sbits], dtype=np.uint16)
        with np.errstate(over="ignore", invalid="ignore"):
            ref = np.ldexp(s16, E).astype(np.float16)
            ref = (-ref if sign else ref).view(np.uint16)
        nan = np.isnan(s16)
        # definition == numpy for every non-NaN scale (rounding, subnormals, overflow included)
        assert np.array_equal(d[~nan], ref[~nan])
        # recipe == definition everywhere inside the domain ...
        assert np.array_equal(r[in_dom], d[in_dom])
        dom_flag = np.array([oracle.scale_in_domain(int(b), bits) for b in sbits])
        assert np.array_equal(dom_flag, in_dom)
        # ... and the mantissa is never touched, the exponent field moves by E, bit 15 is the sign
        assert np.array_equal(r[in_dom] & 0x3FF, sbits[in_dom] & 0x3FF)
        assert np.array_equal(((r[in_dom] >> 10) & 31).astype(int) - ((sbits[in_dom] >> 10) & 31), np.full(in_dom.sum(), E))
        assert np.all((r[in_dom] >> 15) == sign)
    # outside the domain they differ somewhere (zero and subnormal scales, E > 0)
    if qmax > 0:
        assert oracle.decode_def(1, 0x0001, bits) != oracle.decode_bits(1, 0x0001, bits)
        assert oracle.decode_def(1, 0x0000, bits) == 0 and oracle.decode_bits(1, 0x0000, bits) == 0x0400


def test_shift_direction_reading():
    # s = 1.0, 3-bit code 111: 0x3C00 + ((1<<5 | 3) << 10) = 0xC800 = -8 = -(2^3) * s
    assert oracle.decode_bits(0b111, 0x3C00, 3) == 0xC800
    assert oracle.half_to_double(0xC800) == -8.0


def test_check_scales_counts():
    s = np.array([0x3C00, 0x0000, 0x03FF, 0x0400, 0x6FFF, 0x7000, 0xBC00, 0x7C00, 0x7E00], dtype=np.uint16)
    # bits=3: exponent field must be 1..27 and sign 0
    assert oracle.check_scales(s, 3) == 6
    # bits=2: 1..29
    assert oracle.check_scales(s, 2) == 5


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_int_decode_brute_force(bits):
    rng = np.random.default_rng(11 + bits)
    S = np.concatenate([rng.uniform(1e-3, 0.1, 300), [1.0, 0.5, 6.1e-5, 3.0e-7]]).astype(np.float16)
    for q in range(2 ** bits):
        for Z in range(-(2 ** bits - 1), 1):
            zb = int(np.float16(Z).view(np.uint16))
            ref = ((q + Z) * S.astype(np.float64)).astype(np.float16).view(np.uint16)
            got = np.array([oracle.int_decode(q, int(s), zb) for s in S.view(np.uint16)], dtype=np.uint16)
            assert np.array_equal(got, ref)
            if q + Z == 0:
                assert np.all(got == 0)           # +0 exactly
    # S = 1 gives the small integers exactly
    one = int(np.float16(1.0).view(np.uint16))
    for q in range(2 ** bits):
        assert oracle.half_to_double(oracle.int_decode(q, one, int(np.float16(-3).view(np.uint16)))) == q - 3
