"""GPU parity of the exponent form of the PoT GEMV (Sec. 4.2, additivity of exponents: the
scale applied once per group, integer inner sums) against the oracle, through pot_gemv and
pot_gemv_batch on shapes large enough to be served by it: ragged group counts, several row
tiles per workgroup, the sixteen-wavefront variant for long rows, both group sizes, and
activation vectors that stress the fixed-point conversion of x."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import REL_TOL, dev, host_bits, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def potq():
    import paper_2507_11959_amd as p
    return p


def _threads():
    import os
    return min(16, len(os.sched_getaffinity(0)))


def _x(kind: str, K: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(K).astype(np.float32)
    if kind == "outlier":            # a few channels 200x the rest, as activation outliers are
        x[rng.choice(K, 8, replace=False)] *= 200.0
    elif kind == "tiny":
        x *= 1e-4
    elif kind == "wide":             # 30 binades of dynamic range: small entries fall off the fixed-point grid
        x *= np.exp2(rng.integers(-20, 10, K)).astype(np.float32)
    elif kind == "subnormal":
        x *= 3e-7
    elif kind == "zero":
        x[:] = 0.0
    elif kind == "largest":          # the largest finite fp16 among ordinary entries
        x[rng.choice(K, 4, replace=False)] = 65504.0
    return x.astype(np.float16)


def _check(potq, N, K, bits, group, kind="normal", seed=0):
    assert potq.potq_gemv_exponent_form(N, K, bits), "shape is meant to take the exponent form"
    packed, S = workloads.pot_matrix(6, seed, N, K, bits, group)
    x = _x(kind, K, seed)
    tiled = potq.potq_repack(dev(packed), K, bits)
    got = host_bits(potq.pot_gemv(tiled, dev(S), dev(x), K, bits, group))
    want = oracle.gemm(packed, S, None, x[None, :], K, bits, group, nthreads=_threads())[0]
    _assert_close(got, want, K, (N, K, bits, group, kind))
    return got, want


def _assert_close(got, want, K, what):
    """The fused kernels' gate, |y - ref| <= 2e-3 * max(|ref|, floor), with the two ends of the fp16
    range treated as what they are: a sum beyond the range is the same infinity on both sides, and
    an output below the normal range (|ref| < 2^-14, which tiny or subnormal activations produce)
    is a multiple of 2^-24, so one such quantum is allowed on top -- there it is a relative error
    far above any tolerance and means nothing."""
    from gpu_util import floor_fraction
    w = want.view(np.float16).astype(np.float64)
    g = got.view(np.float16).astype(np.float64)
    finite = np.isfinite(w)
    assert np.array_equal(got[~finite], want[~finite]), what
    w, g = w[finite], g[finite]
    if w.size == 0:
        return
    floor = np.sqrt(np.mean(w * w)) * floor_fraction(K)
    allowed = REL_TOL * np.maximum(np.abs(w), floor) + np.where(np.abs(w) < 2.0 ** -14, 2.0 ** -24, 0.0)
    excess = np.abs(g - w) - allowed
    assert excess.max() <= 0.0, (what, float((np.abs(g - w) / np.maximum(np.abs(w), max(floor, 1e-300))).max()))


@pytest.mark.parametrize("N,K,bits,group", [
    (15904, 4224, 3, 128),     # 33 groups: one wavefront has a second round; 994 tiles over 497 workgroups
    (8208, 8192, 2, 128),      # 513 tiles: the last workgroup has one tile fewer
    (9600, 7040, 3, 64),       # group size 64, 55 groups
    (4112, 16384, 2, 64),      # long rows: sixteen wavefronts, two tiles at a time, odd number of tiles
    (2320, 30464, 3, 128),     # long rows: the digits of x take 134 KB of LDS
])
def test_shapes(potq, N, K, bits, group):
    _check(potq, N, K, bits, group)


@pytest.mark.parametrize("kind", ["outlier", "tiny", "wide", "subnormal", "zero", "largest"])
def test_activation_ranges(potq, kind):
    got, want = _check(potq, 8192, 8192, 3, 128, kind, seed=3)
    if kind == "zero":
        assert not got.any()


def _same_non_finite(got_bits, want_bits, what):
    g = got_bits.view(np.float16).astype(np.float64)
    w = want_bits.view(np.float16).astype(np.float64)
    assert not np.isfinite(w).any(), what              # every row meets the non-finite activation
    assert np.array_equal(np.isnan(g), np.isnan(w)), what
    inf = np.isinf(w)
    assert np.array_equal(g[inf], w[inf]), what         # the same sign of infinity


@pytest.mark.parametrize("N,K,bits,group", [(8192, 8192, 3, 128), (8208, 8192, 2, 64)])
@pytest.mark.parametrize("case", ["one_inf", "two_inf_same_sign", "inf_both_signs", "nan", "inf_and_nan"])
def test_non_finite_activations_follow_the_definition(potq, N, K, bits, group, case):
    """An infinity among the activations reaches every row with the sign its weight gives it: rows whose
    infinite terms agree come out as that infinity, the others as NaN; a NaN makes every row NaN.  The
    result is the oracle's whichever kernel serves the matrix."""
    packed, S = workloads.pot_matrix(6, 9, N, K, bits, group)
    x = _x("normal", K, 9)
    if case == "one_inf":
        x[17] = np.float16(np.inf)
    elif case == "two_inf_same_sign":
        x[17] = x[K - 3] = np.float16(-np.inf)
    elif case == "inf_both_signs":
        x[5], x[4100], x[K - 1] = np.float16(np.inf), np.float16(-np.inf), np.float16(np.inf)
    elif case == "nan":
        x[4242] = np.float16(np.nan)
    else:
        x[0], x[1] = np.float16(np.inf), np.float16(np.nan)
    tiled = potq.potq_repack(dev(packed), K, bits)
    got = host_bits(potq.pot_gemv(tiled, dev(S), dev(x), K, bits, group))
    want = oracle.gemm(packed, S, None, x[None, :], K, bits, group, nthreads=_threads())[0]
    _same_non_finite(got, want, (N, K, bits, group, case))
    if case == "one_inf":
        assert np.isinf(want.view(np.float16)).all() and len(np.unique(want)) == 2     # both signs occur
    if case in ("two_inf_same_sign", "inf_both_signs"):     # the weights' signs decide, row by row
        w = want.view(np.float16)
        assert np.isnan(w).any() and np.isinf(w).any()


def test_non_finite_activations_with_two_to_four_tokens(potq):
    """The multi-vector kernel: one vector with an infinity, one with a NaN, two ordinary ones."""
    M, N, K, bits = 4, 17920, 6656, 3
    assert potq.potq_gemv_exponent_form(N, K, bits)
    packed, S = workloads.pot_matrix(6, 58, N, K, bits, 128)
    X = np.stack([_x("normal", K, 70 + m) for m in range(M)])
    X[1, 33] = np.float16(-np.inf)
    X[2, 6000] = np.float16(np.nan)
    tiled = potq.potq_repack(dev(packed), K, bits)
    Y = host_bits(potq.pot_gemm(tiled, dev(S), dev(X), K, bits))
    rows = np.unique(np.concatenate([[0, 15, 16, N - 1], np.arange(5, N, 61)]))
    want = oracle.gemm(packed[rows], S[rows], None, X, K, bits, 128, nthreads=_threads())
    for m in (1, 2):
        _same_non_finite(Y[m][rows], want[m], ("tokens", m))
    for m in (0, 3):
        e, nw, nfloor = rel_err(Y[m][rows], want[m], K)
        assert e <= REL_TOL, (m, e, nw, nfloor)


@pytest.mark.parametrize("bits", [2, 3])
def test_batch_sharing_x(potq, bits):
    K, rows = 4096, (11008, 5504, 16)          # 16 528 rows together: served in the exponent form
    assert potq.potq_gemv_batch_exponent_form(len(rows), K, bits)
    x = _x("outlier", K, 11)
    mats, refs = [], []
    for i, N in enumerate(rows):
        packed, S = workloads.pot_matrix(6, 20 + i, N, K, bits, 128)
        mats.append((potq.potq_repack(dev(packed), K, bits), dev(S)))
        refs.append(oracle.gemm(packed, S, None, x[None, :], K, bits, 128, nthreads=_threads())[0])
    ys = potq.pot_gemv_batch(mats, dev(x), K, bits)
    for y, want in zip(ys, refs):
        e, nw, nfloor = rel_err(host_bits(y), want, K)
        assert e <= REL_TOL, (bits, e, nw, nfloor)


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("bits", [2, 3])
@pytest.mark.parametrize("K", [4096, 5120, 16384])
def test_small_batches_sharing_x(potq, K, bits, group):
    """Matrices that share x take the exponent form at every size: the largest batch the entry
    point accepts, of matrices of one to thirteen row tiles (fewer tiles than workgroups), and a
    batch of two single-tile matrices."""
    assert potq.potq_gemv_batch_exponent_form(16, K, bits)
    x = _x("normal", K, 40 + bits)
    for rows in ([16 * (1 + (5 * i) % 13) for i in range(16)], [16, 16]):
        mats, refs = [], []
        for i, N in enumerate(rows):
            packed, S = workloads.pot_matrix(6, 60 + i + 20 * (group == 64), N, K, bits, group)
            mats.append((potq.potq_repack(dev(packed), K, bits), dev(S)))
            refs.append(oracle.gemm(packed, S, None, x[None, :], K, bits, group, nthreads=_threads())[0])
        ys = potq.pot_gemv_batch(mats, dev(x), K, bits, group)
        for i, (y, want) in enumerate(zip(ys, refs)):
            e, nw, nfloor = rel_err(host_bits(y), want, K)
            assert e <= REL_TOL, (K, bits, group, len(rows), i, e, nw, nfloor)


def test_gemm_with_one_token_takes_the_same_path(potq):
    N, K, bits = 8192, 8192, 3
    packed, S = workloads.pot_matrix(6, 30, N, K, bits, 128)
    x = _x("normal", K, 30)
    tiled = potq.potq_repack(dev(packed), K, bits)
    y1 = host_bits(potq.pot_gemv(tiled, dev(S), dev(x), K, bits))
    y2 = host_bits(potq.pot_gemm(tiled, dev(S), dev(x[None, :]), K, bits))[0]
    assert np.array_equal(y1, y2)


@pytest.mark.parametrize("M,N,K,bits", [
    (2, 8208, 8192, 3),        # two tokens: eight wavefronts, two workgroups' digits share a compute unit's LDS
    (2, 10240, 13824, 2),      # two tokens, long rows: sixteen wavefronts
    (3, 16400, 8192, 3),       # three tokens in the four-vector kernel (the fourth counts as zero), 1025 row tiles
    (4, 17920, 6656, 2),       # four tokens, ragged group count (52)
])
def test_two_to_four_tokens(potq, M, N, K, bits):
    """pot_gemm with two to four tokens on tall, large matrices runs the exponent form with one
    MFMA per vector and step; every vector has its own fixed-point exponent (rows of X differ
    in scale by up to 2^12 here)."""
    rng = np.random.default_rng(100 + M)
    packed, S = workloads.pot_matrix(6, 50 + M, N, K, bits, 128)
    X = np.stack([_x("outlier" if m % 2 else "normal", K, 60 + m).astype(np.float32) * 2.0 ** (-4 * m)
                  for m in range(M)]).astype(np.float16)
    tiled = potq.potq_repack(dev(packed), K, bits)
    Y = potq.pot_gemm(tiled, dev(S), dev(X), K, bits)
    rows = np.unique(np.concatenate([[0, 15, 16, N - 17, N - 1], rng.integers(0, N, 400)]))
    want = oracle.gemm(packed[rows], S[rows], None, X, K, bits, 128, nthreads=_threads())
    got = host_bits(Y[:, torch.from_numpy(rows).to("cuda:0")].contiguous())
    for m in range(M):                       # per token: the rows differ in scale, and so does the error floor
        e, nw, nfloor = rel_err(got[m], want[m], K)
        assert e <= REL_TOL, (M, N, K, bits, m, e, nw, nfloor)
    assert bool(torch.isfinite(Y).all())
