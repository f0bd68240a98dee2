"""Pins for the oracle's Step 1 scale search (Sec. 3.2, Algorithm 1): hand-derived
closed-form cases, and the paper's literal formula evaluated in numpy float64."""
import numpy as np
import pytest

import oracle
import workloads


def _literal(W64, s, qmax):
    """E = clamp(round(log2(|W|/s)), 0, qmax) and the reconstruction, as printed (float64)."""
    with np.errstate(divide="ignore"):
        E = np.clip(np.rint(np.log2(np.abs(W64) / s)), 0, qmax)
    E = np.where(W64 == 0, 0, E)
    return E, np.where(W64 < 0, -1.0, 1.0) * s * 2.0 ** E


def test_closed_form_equal_magnitudes():
    # |w| = a everywhere.  b=3: s0 = a/7; zero error needs s*2^E = a, on the grid only at 1.75 (E=2).
    # b=2: s0 = a; zero error at 0.5 (E=1) and 1.0 (E=0); the strict '<' keeps the first, 0.5.
    a = np.float16(0.3)
    W = np.tile(np.array([a, -a], np.float16), (3, 128))
    c, s, i = oracle.pot_quantize(W, 3, 128, want_index=True)
    assert np.all(i == 175) and np.all(c[:, 0::2] == 2) and np.all(c[:, 1::2] == 6)
    assert np.all(s.view(np.float16) == np.float16(float(a) / 4))
    c, s, i = oracle.pot_quantize(W, 2, 128, want_index=True)
    assert np.all(i == 50) and np.all(c[:, 0::2] == 1) and np.all(c[:, 1::2] == 3)
    assert np.all(s.view(np.float16) == np.float16(float(a) / 2))


def test_two_level_group_is_reproduced_exactly():
    # weights already on a PoT grid {±v, ±2v, ±4v, ±8v}: the search must find a zero-error scale
    v = 0.0078125  # 2^-7
    rng = np.random.default_rng(0)
    lev = rng.integers(0, 4, size=(4, 256))
    sg = rng.choice([-1.0, 1.0], size=(4, 256))
    lev[:, 0] = 3          # make sure the top level occurs in every group
    lev[:, 128] = 3
    W = (sg * v * 2.0 ** lev).astype(np.float16)
    c, s, i = oracle.pot_quantize(W, 3, 128, want_index=True)
    # s0 = 8v/7, zero error needs s = v = s0 * 0.875: not on the grid; but 2v = s0*1.75 cannot hold level v.
    # So the optimum is not exact here; check instead that the reconstruction beats the naive b = 1.
    Wd = oracle.pot_dequant(oracle.pack_codes(c, 3), s, 256, 3, 128).view(np.float16).astype(np.float64)
    err = ((W.astype(np.float64) - Wd) ** 2).reshape(4, 2, 128).sum(axis=2)
    s_naive = (8 * v / 7)
    _, Wn = _literal(W.astype(np.float64), s_naive, 3)
    err_naive = ((W.astype(np.float64) - Wn) ** 2).reshape(4, 2, 128).sum(axis=2)
    assert np.all(err <= err_naive * (1 + 1e-3))


@pytest.mark.parametrize("bits,group", [(2, 128), (3, 128), (3, 64), (4, 128)])
def test_against_the_literal_formula_in_float64(bits, group):
    qmax = 2 ** (bits - 1) - 1
    N, K = 48, 1024
    W = workloads.weights_f16(42 + bits + group, N, K)
    codes, scales, idx = oracle.pot_quantize(W, bits, group, want_index=True)
    W64 = W.astype(np.float64).reshape(N, K // group, group)
    wmax = np.abs(W64).max(axis=2)
    # the candidates as they would be stored (Sec. 4.2: the scale is FP16): s0 * b_i in binary32, rounded once
    # to binary16 by numpy, clamped into the exact domain of the de-quantisation recipe
    s0 = wmax.astype(np.float32) / np.float32(2 ** qmax - 1)
    mult = np.arange(1, 201, dtype=np.float32) * np.float32(0.01)
    lo = np.float16(2.0 ** -14)
    hi = np.array([((30 - qmax) << 10) | 0x3FF], dtype=np.uint16).view(np.float16)[0]
    cand = np.clip((s0[..., None] * mult).astype(np.float16), lo, hi)                  # (N, groups, 200) fp16
    # Q(i) for every candidate by the printed formula, in float64
    Q = np.empty((N, K // group, 200))
    for j in range(200):
        _, Wq = _literal(W64, cand[..., j].astype(np.float64)[..., None], qmax)
        Q[..., j] = ((W64 - Wq) ** 2).sum(axis=2)
    qmin = Q.min(axis=2)
    chosen = np.take_along_axis(Q, (idx - 1)[..., None], axis=2)[..., 0]
    # the oracle's choice is optimal up to binary32 rounding of the error sums
    assert np.all(chosen <= qmin * (1 + 1e-5))
    # and it is the very same index, except where two candidates tie within that rounding (the float64
    # evaluation then cannot tell which one binary32 prefers; neighbouring multipliers that round to the same
    # fp16 scale tie exactly, and both sides keep the first); such ties are rare
    same = np.argmin(Q, axis=2) + 1 == idx
    assert np.all(same | (chosen <= qmin * (1 + 1e-6)))
    assert same.mean() >= 0.99
    # the stored scale is the chosen candidate
    stored = np.take_along_axis(cand, (idx - 1)[..., None], axis=2)[..., 0]
    assert np.array_equal(scales, stored.view(np.uint16))
    # the codes are the printed formula's codes under the stored scale, except within rounding of a threshold
    s_stored = stored.astype(np.float64)
    E_lit, W_lit = _literal(W64, s_stored[..., None], qmax)
    E = (codes & (2 ** (bits - 1) - 1)).reshape(N, K // group, group)
    ratio = np.abs(W64) / s_stored[..., None]
    with np.errstate(divide="ignore"):
        frac = np.abs(np.log2(np.where(ratio > 0, ratio, 1.0)) % 1.0 - 0.5)
    near_threshold = frac < 1e-5
    assert np.all((E == E_lit) | near_threshold)
    # and what pot_dequant rebuilds from (codes, scale) is that reconstruction, bit for bit
    Wd = oracle.pot_dequant(oracle.pack_codes(codes, bits), scales, K, bits, group).view(np.float16)
    Wd = Wd.astype(np.float64).reshape(N, K // group, group)
    assert np.array_equal(Wd[~near_threshold], W_lit[~near_threshold])
    sign = (codes >> (bits - 1)).reshape(N, K // group, group)
    assert np.array_equal(sign == 1, W64 < 0)
    # never worse than the naive multiplier b = 1 (i = 100)
    assert np.all(chosen <= Q[..., 99] * (1 + 1e-6))
    assert oracle.check_scales(scales, bits) == 0
    # threads do not change the result
    c2, s2 = oracle.pot_quantize(W, bits, group, nthreads=4)
    assert np.array_equal(c2, codes) and np.array_equal(s2, scales)


def test_degenerate_groups():
    W = np.zeros((2, 256), np.float16)
    W[0, 130] = -0.5                      # second group of row 0: one non-zero
    W[1, :128] = 6e-8                     # subnormal fp16 everywhere: scale clamps to 2^-14
    c, s, i = oracle.pot_quantize(W, 3, 128, want_index=True)
    assert np.all(c[0, :128] == 0) and s[0, 0] == 0x0400          # all-zero group: E = 0, smallest normal scale
    assert c[0, 130] >> 2 == 1 and np.all(c[0, 128:130] >> 2 == 0)
    assert s[1, 0] == 0x0400 and np.all(s >= 0x0400)
    assert oracle.check_scales(s, 3) == 0
    # One weight of -0.5 among 127 zeros.  PoT has no zero level, so the zeros cost 127 s^2 and the
    # lone weight (0.5 - 8 s)^2: the continuous optimum is s = 4/191 = 0.02094 = 0.2932 * s0 with
    # s0 = 0.5/7; of the two neighbouring grid points Q(0.29) = 0.16624 < Q(0.30) = 0.16628.
    assert i[0, 1] == 29 and c[0, 130] == 0b111
    Wd = oracle.pot_dequant(oracle.pack_codes(c, 3), s, 256, 3, 128).view(np.float16)
    assert abs(float(Wd[0, 130]) + 8 * 0.29 * 0.5 / 7) < 2e-4
