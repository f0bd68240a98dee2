"""GPU parity tests: the HIP library, called through the C ABI, against the CPU
oracle on the same seeded inputs.  Dequant is compared bit for bit; the fused
GEMV / GEMM within the stated relative tolerance, and bit for bit wherever the
result is a single term (one-hot activations)."""
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


# shapes: several 2048-weight wavefront chunks plus a ragged tail; one-group and one-row cases
DEQ_SHAPES = [(37, 640), (1, 128), (3, 128), (16, 2048), (5, 11008), (129, 4096)]


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("N,K", DEQ_SHAPES)
def test_pot_dequant_bit_exact(potq, bits, group, N, K):
    packed = workloads.packed_codes(11 * N + K + bits, N, K, bits)
    scales = workloads.pot_scales(13 * N + K + group, N, K, group)
    want = oracle.pot_dequant(packed, scales, K, bits, group, nthreads=4)
    got = host_bits(potq.pot_dequant(dev(packed), dev(scales), K, bits, group))
    assert got.shape == want.shape
    assert np.array_equal(got, want)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("N,K", DEQ_SHAPES)
def test_int_dequant_bit_exact(potq, bits, group, N, K):
    packed = workloads.packed_codes(17 * N + K + bits, N, K, bits)
    S, Z = workloads.int_scales_zeros(19 * N + K + group, N, K, bits, group)
    want = oracle.int_dequant(packed, S, Z, K, bits, group, nthreads=4)
    got = host_bits(potq.int_dequant(dev(packed), dev(S), dev(Z), K, bits, group))
    assert np.array_equal(got, want)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("is_int", [False, True])
def test_dequant_batch_equals_single_calls_and_oracle(potq, bits, is_int):
    # several matrices of different sizes (ragged tails, one empty) in one launch
    shapes = [(37, 640), (1, 128), (0, 256), (16, 2048), (129, 4096), (5, 11008), (64, 128)]
    G = 128
    mats, wants = [], []
    for i, (N, K) in enumerate(shapes):
        packed = workloads.packed_codes(31 * i + bits, N, K, bits)
        if is_int:
            S, Z = workloads.int_scales_zeros(37 * i + bits, N, K, bits, G)
            want = oracle.int_dequant(packed, S, Z, K, bits, G, nthreads=4)
        else:
            S, Z = workloads.pot_scales(41 * i + bits, N, K, G), None
            want = oracle.pot_dequant(packed, S, K, bits, G, nthreads=4)
        out = torch.full((N, K), 7.0, dtype=torch.float16, device="cuda:0")
        if is_int:
            mats.append((dev(packed), dev(S), dev(Z), out, K))
        else:
            mats.append((dev(packed), dev(S), out, K))
        wants.append(want)
    if is_int:
        potq.int_dequant_batch(mats, bits, G)
    else:
        potq.pot_dequant_batch(mats, bits, G)
    for m, want in zip(mats, wants):
        got = host_bits(m[-2])
        assert np.array_equal(got, want)
    # too many matrices is an error, not a crash
    from paper_2507_11959_amd import binding
    arr = binding.make_batch([(m[0], m[1], None, m[-2], m[-1], bits) for m in mats if m[0].numel()])
    assert binding.raw().pot_dequant_batch(arr, 17, bits, G, None) == 4
    assert binding.raw().pot_dequant_batch(None, 3, bits, G, None) == 1
    assert binding.raw().pot_dequant_batch(None, 0, bits, G, None) == 0


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("count", [8, 9, 16])
def test_dequant_batch_full_table(potq, bits, count):
    # up to the largest batch the table holds: equal sizes, empties between them, one-workgroup
    # and many-workgroup matrices, so that every slot of the lookup decides some piece
    base = [(24, 4096), (0, 128), (3, 128), (24, 4096), (200, 2048), (1, 256), (0, 512), (65, 1152),
            (24, 4096), (7, 128), (0, 128), (130, 4096), (2, 11008), (24, 4096), (1, 128), (33, 640)]
    shapes = base[:count]
    G = 128
    mats, wants = [], []
    for i, (N, K) in enumerate(shapes):
        packed = workloads.packed_codes(53 * i + bits, N, K, bits)
        S = workloads.pot_scales(59 * i + bits, N, K, G)
        wants.append(oracle.pot_dequant(packed, S, K, bits, G, nthreads=4))
        mats.append((dev(packed), dev(S), torch.full((N, K), 7.0, dtype=torch.float16, device="cuda:0"), K))
    potq.pot_dequant_batch(mats, bits, G)
    for m, want in zip(mats, wants):
        assert np.array_equal(host_bits(m[-2]), want)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_pot_dequant_structured_pattern(potq, bits):
    # code(n,k) = (n + k) mod 2^b, scale(n,g) = 2^((n+g) mod 8 - 8): index mix-ups change the output
    N, K, G = 40, 1024, 128
    n = np.arange(N)[:, None]
    codes = ((n + np.arange(K)[None, :]) % 2 ** bits).astype(np.uint8)
    scales = (2.0 ** (((n + np.arange(K // G)[None, :]) % 8) - 8)).astype(np.float16)
    packed = oracle.pack_codes(codes, bits)
    want = oracle.pot_dequant(packed, scales, K, bits, G)
    got = host_bits(potq.pot_dequant(dev(packed), dev(scales), K, bits, G))
    assert np.array_equal(got, want)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_pot_dequant_any_scale_pattern_is_the_bit_recipe(potq, bits):
    # outside the exact domain the library's result is defined as the 16-bit wrap-around add
    N, K, G = 64, 1024, 128
    rng = np.random.default_rng(bits)
    scales = rng.integers(0, 65536, size=(N, K // G), dtype=np.uint16)
    packed = workloads.packed_codes(5, N, K, bits)
    want = oracle.pot_dequant(packed, scales, K, bits, G, use_bit_recipe=True)
    got = host_bits(potq.pot_dequant(dev(packed), dev(scales), K, bits, G))
    assert np.array_equal(got, want)
    bad = oracle.check_scales(scales, bits)
    assert 0 < bad < scales.size
    assert potq.pot_check_scales(dev(scales), bits) == bad
    assert potq.pot_check_scales(dev(workloads.pot_scales(1, N, K)), bits) == 0


def test_int_dequant_all_zero_points(potq):
    # every (q, Z) pair with sampled scales, including S = 1 (exact small integers)
    for bits in (2, 3):
        L = 2 ** bits - 1
        N, K, G = 16 * (L + 1), 128, 128
        codes = np.tile(np.arange(K) % (L + 1), (N, 1)).astype(np.uint8)
        packed = oracle.pack_codes(codes, bits)
        Z = np.repeat(-np.arange(L + 1), 16).astype(np.float16)[:, None]
        rng = np.random.default_rng(3)
        S = rng.uniform(1e-3, 0.1, size=(N, 1)).astype(np.float16)
        S[::16] = 1.0
        want = oracle.int_dequant(packed, S, Z, K, bits, G)
        got = host_bits(potq.int_dequant(dev(packed), dev(S), dev(Z), K, bits, G))
        assert np.array_equal(got, want)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", [(16, 128), (48, 640), (256, 4096)])
def test_repack_round_trip_and_permutation(potq, bits, N, K):
    packed = workloads.packed_codes(23 + N + bits, N, K, bits)
    d = dev(packed)
    tiled = potq.potq_repack(d, K, bits, potq.LAYOUT_TILE16)
    back = potq.potq_repack(tiled, K, bits, potq.LAYOUT_CANONICAL)
    assert torch.equal(back, d)
    assert tiled.numel() == d.numel()
    # a permutation of bits: same population count, and (for random input) not the identity
    t = tiled.cpu().numpy()
    assert np.unpackbits(t).sum() == np.unpackbits(packed).sum()
    assert not np.array_equal(t.ravel(), packed.ravel())


def _gemv_inputs(seed, N, K, bits, is_int, group=128):
    packed = workloads.packed_codes(seed, N, K, bits)
    if is_int:
        S, Z = workloads.int_scales_zeros(seed + 3, N, K, bits, group)
    else:
        S, Z = workloads.pot_scales(seed + 1, N, K, group), None
    return packed, S, Z


def _run_gemm(potq, packed, S, Z, X, K, bits, use_workspace=True, group=128):
    tiled = potq.potq_repack(dev(packed), K, bits)
    ws = potq.gemm_workspace(X.shape[0], packed.shape[0], K, bits) if use_workspace else None
    if X.shape[0] == 1:
        if Z is None:
            y = potq.pot_gemv(tiled, dev(S), dev(X[0]), K, bits, group)
        else:
            y = potq.int_gemv(tiled, dev(S), dev(Z), dev(X[0]), K, bits, group)
        return host_bits(y)[None, :]
    if Z is None:
        return host_bits(potq.pot_gemm(tiled, dev(S), dev(X), K, bits, group, workspace=ws))
    return host_bits(potq.int_gemm(tiled, dev(S), dev(Z), dev(X), K, bits, group, workspace=ws))


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", [(16, 128), (48, 640), (272, 4096), (64, 11008)])
def test_gemv_one_hot_gives_exact_columns(potq, bits, N, K, is_int):
    packed, S, Z = _gemv_inputs(100 + N + bits, N, K, bits, is_int)
    W = oracle.int_dequant(packed, S, Z, K, bits, 128) if is_int else oracle.pot_dequant(packed, S, K, bits, 128)
    rng = np.random.default_rng(N + K)
    ks = sorted(set([0, 1, 2, 3, 31, 32, 127, K - 128, K - 1] + list(rng.integers(0, K, 24))))
    for k in ks:
        X = np.zeros((1, K), np.float16)
        X[0, k] = 1.0
        y = _run_gemm(potq, packed, S, Z, X, K, bits)[0]
        assert np.array_equal(y, W[:, k]), k


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", [(16, 128), (48, 640), (272, 4096), (64, 11008), (1024, 8192)])
def test_gemv_vs_oracle(potq, bits, N, K, is_int):
    packed, S, Z = _gemv_inputs(200 + N + bits, N, K, bits, is_int)
    X = workloads.activations(300 + K, 1, K)
    want = oracle.gemm(packed, S, Z, X, K, bits, 128, nthreads=8)
    got = _run_gemm(potq, packed, S, Z, X, K, bits)
    e, nw, nfloor = rel_err(got, want, K)
    assert e <= REL_TOL, (e, nw, nfloor)


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("M,N,K", [(1, 48, 640), (1, 272, 4096), (1, 32, 11008), (16, 80, 1280), (70, 64, 2560),
                                   (256, 144, 1024)])
def test_group_size_64_in_fused_kernels(potq, bits, M, N, K, is_int):
    # Sec. 3.1 names 64 as the other group size: two scales per 128-column tile row
    packed, S, Z = _gemv_inputs(1100 + M + N + bits, N, K, bits, is_int, group=64)
    assert S.shape == (N, K // 64)
    X = workloads.activations(1200 + M, M, K)
    want = oracle.gemm(packed, S, Z, X, K, bits, 64, nthreads=8)
    got = _run_gemm(potq, packed, S, Z, X, K, bits, group=64)
    e, nw, nfloor = rel_err(got, want, K)
    assert e <= REL_TOL, (e, nw, nfloor)
    # exact columns through one-hot activations, on both halves of a tile row
    W = oracle.int_dequant(packed, S, Z, K, bits, 64) if is_int else oracle.pot_dequant(packed, S, K, bits, 64)
    ks = [0, 63, 64, 127, 128, K - 65, K - 1]
    E = np.zeros((len(ks) if M > 1 else 1, K), np.float16)
    if M > 1:
        E[np.arange(len(ks)), ks] = 1.0
        assert np.array_equal(_run_gemm(potq, packed, S, Z, E, K, bits, group=64), W[:, ks].T)
    else:
        for k in ks:
            E[:] = 0
            E[0, k] = 1.0
            assert np.array_equal(_run_gemm(potq, packed, S, Z, E, K, bits, group=64)[0], W[:, k]), k


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("bits,group", [(3, 128), (2, 128), (3, 64), (4, 128)])
def test_gemv_batch_shared_activation_equals_single_calls(potq, bits, group, is_int):
    K = 2560
    Ns = [64, 16, 272, 0, 48]
    x = workloads.activations(1300 + bits, 1, K)
    dx = dev(x[0])
    mats, singles = [], []
    for i, N in enumerate(Ns):
        packed, S, Z = _gemv_inputs(1400 + 7 * i + bits, N, K, bits, is_int, group)
        tiled = potq.potq_repack(dev(packed), K, bits) if N else torch.empty((0, K * bits // 8), dtype=torch.uint8,
                                                                               device="cuda:0")
        if is_int:
            mats.append((tiled, dev(S), dev(Z)))
            singles.append(potq.int_gemv(tiled, dev(S), dev(Z), dx, K, bits, group) if N else None)
        else:
            mats.append((tiled, dev(S)))
            singles.append(potq.pot_gemv(tiled, dev(S), dx, K, bits, group) if N else None)
        if N:
            want = oracle.gemm(packed, S, Z, x, K, bits, group, nthreads=8)[0]
            e, nw, nfloor = rel_err(host_bits(singles[-1]), want, K)
            assert e <= REL_TOL
    ys = potq.int_gemv_batch(mats, dx, K, bits, group) if is_int else potq.pot_gemv_batch(mats, dx, K, bits, group)
    for y, single in zip(ys, singles):
        if single is not None:
            assert torch.equal(y, single)


def test_gemv_all_ones_zero_codes(potq):
    N, K = 32, 1024
    scales = (2.0 ** -(np.arange(K // 128) % 4)[None, :] * np.ones((N, 1))).astype(np.float16)
    packed = np.zeros((N, K * 3 // 8), np.uint8)
    y = _run_gemm(potq, packed, scales, None, np.ones((1, K), np.float16), K, 3)[0]
    assert np.all(y.view(np.float16).astype(np.float64) == 128 * scales.astype(np.float64).sum(axis=1))


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("M", [2, 16, 33, 70, 256])
def test_gemm_vs_oracle(potq, bits, M, is_int):
    N, K = 80, 1280
    packed, S, Z = _gemv_inputs(400 + M + bits, N, K, bits, is_int)
    X = workloads.activations(500 + M, M, K)
    want = oracle.gemm(packed, S, Z, X, K, bits, 128, nthreads=8)
    got = _run_gemm(potq, packed, S, Z, X, K, bits)
    assert got.shape == (M, N)
    e, nw, nfloor = rel_err(got, want, K)
    assert e <= REL_TOL, (e, nw, nfloor)


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("M,N,K", [(16, 64, 4096), (8, 48, 11008), (40, 128, 2560), (64, 32, 8192)])
def test_gemm_split_k_matches_oracle_and_is_reproducible(potq, bits, M, N, K):
    # few tokens and few rows: the workspace path splits K over several workgroups
    packed, S, Z = _gemv_inputs(700 + M + bits, N, K, bits, False)
    X = workloads.activations(800 + M, M, K)
    want = oracle.gemm(packed, S, None, X, K, bits, 128, nthreads=8)
    a = _run_gemm(potq, packed, S, None, X, K, bits, use_workspace=True)
    b = _run_gemm(potq, packed, S, None, X, K, bits, use_workspace=True)
    c = _run_gemm(potq, packed, S, None, X, K, bits, use_workspace=False)
    assert np.array_equal(a, b)                       # fixed summation order: bit-identical reruns
    for got in (a, c):
        e, nw, nfloor = rel_err(got, want, K)
        assert e <= REL_TOL, (e, nw, nfloor)
    # a workspace too small for two splits is accepted and simply not used
    tiled = potq.potq_repack(dev(packed), K, bits)
    tiny = torch.empty((64,), dtype=torch.uint8, device="cuda:0")
    d = host_bits(potq.pot_gemm(tiled, dev(S), dev(X), K, bits, workspace=tiny))
    assert np.array_equal(d, c)


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_gemm_one_hot_rows_give_exact_columns(potq, bits, is_int):
    N, K, M = 48, 640, 40
    packed, S, Z = _gemv_inputs(600 + bits, N, K, bits, is_int)
    W = oracle.int_dequant(packed, S, Z, K, bits, 128) if is_int else oracle.pot_dequant(packed, S, K, bits, 128)
    ks = np.random.default_rng(9).choice(K, size=M, replace=False)
    X = np.zeros((M, K), np.float16)
    X[np.arange(M), ks] = 1.0
    got = _run_gemm(potq, packed, S, Z, X, K, bits)
    assert np.array_equal(got, W[:, ks].T)


def test_empty_inputs_are_accepted(potq):
    e8 = torch.empty((0,), dtype=torch.uint8, device="cuda:0")
    e16 = torch.empty((0,), dtype=torch.float16, device="cuda:0")
    lib = __import__("paper_2507_11959_amd.binding", fromlist=["raw"]).raw()
    assert lib.pot_dequant(None, None, None, 0, 4096, 3, 128, None) == 0
    assert lib.pot_gemm(None, None, None, None, 0, 16, 128, 3, 128, 1, None, 0, None) == 0
    # K = 0: products over an empty K are zero
    y = torch.full((16,), 7.0, dtype=torch.float16, device="cuda:0")
    assert lib.pot_gemv(None, None, None, y.data_ptr(), 16, 0, 3, 128, 1, None) == 0
    torch.cuda.synchronize()
    assert torch.all(y == 0)
    assert e8.numel() == 0 and e16.numel() == 0


# One case per kernel configuration the GEMM dispatcher can choose (token count x matrix size),
# each with and without a workspace, PoT and uniform, so that no template instance goes untested.
@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("M,N,K", [
    (2, 272, 4096),        # two tokens: the GEMV kernel with one vector per result column
    (3, 64, 5120),         # three tokens in the four-vector instance (fourth vector zero, not stored)
    (4, 48, 4096),         # four tokens
    (2, 32, 11008),        # two tokens, long rows
    (4, 32, 8192),         # four tokens whose vectors do not fit LDS: few-token kernel
    (9, 1024, 2304),       # few-token kernel, 8 wavefronts, ragged last round (18 groups)
    (16, 12304, 384),      # few-token kernel, 16 wavefronts (tall matrix), surplus wavefronts in the last workgroup
    (24, 80, 1280),        # 17-32 tokens, K split inside the workgroup
    (24, 32, 11008),       # 17-32 tokens, long rows: one row tile per wavefront, K split over workgroups
    (30, 8208, 256),       # 17-32 tokens, tall matrix
    (48, 8208, 384),       # 33-64 tokens, tall matrix
    (64, 48, 9216),        # 33-64 tokens, long rows
    (100, 16640, 128),     # more than 64 tokens: narrow 256x64 tile
    (130, 4112, 256),      # narrow tile, ragged token tile
    (1024, 6400, 128),     # wide 256x128 tile (200 workgroups; the narrow tile would need two rounds)
    (2000, 6000, 256),     # tall 384x128 tile (256 workgroups), ragged rows and tokens
    (128, 1024, 5120),     # narrow tile, K split eight ways through the workspace
])
def test_gemm_every_dispatch_configuration(potq, M, N, K, is_int):
    bits = 3
    packed, S, Z = _gemv_inputs(2000 + M + N, N, K, bits, is_int)
    X = workloads.activations(2100 + M, M, K)
    want = oracle.gemm(packed, S, Z, X, K, bits, 128, nthreads=8)
    for use_ws in (True, False):
        got = _run_gemm(potq, packed, S, Z, X, K, bits, use_workspace=use_ws)
        e, nw, nfloor = rel_err(got, want, K)
        assert e <= REL_TOL, (use_ws, e, nw, nfloor)


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("M,N,K", [(128, 1024, 5120), (200, 1024, 2048), (256, 2048, 8192), (130, 4112, 256)])
def test_gemm_plan_does_not_depend_on_spare_workspace(potq, M, N, K, is_int):
    """Above 64 tokens the workspace query returns what the preferred plan needs; a larger workspace must
    not change the plan (same bits), a missing one only removes the K split (same tolerance)."""
    bits = 3
    packed, S, Z = _gemv_inputs(5000 + M + N, N, K, bits, is_int)
    X = workloads.activations(5100 + M, M, K)
    tiled = potq.potq_repack(dev(packed), K, bits)
    need = potq.gemm_workspace(M, N, K, bits)
    spare = torch.empty(((0 if need is None else need.numel()) * 3 + (64 << 20),), dtype=torch.uint8, device="cuda:0")

    def run(ws):
        if is_int:
            return host_bits(potq.int_gemm(tiled, dev(S), dev(Z), dev(X), K, bits, workspace=ws))
        return host_bits(potq.pot_gemm(tiled, dev(S), dev(X), K, bits, workspace=ws))

    preferred, larger, none = run(need), run(spare), run(None)
    assert np.array_equal(preferred, larger)
    want = oracle.gemm(packed, S, Z, X, K, bits, 128, nthreads=8)
    for got in (preferred, none):
        e, nw, nfloor = rel_err(got, want, K)
        assert e <= REL_TOL, (e, nw, nfloor)


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("M,N,K", [
    (1900, 6000, 128),     # tall tile (PoT) / wide tile (uniform), ragged rows and tokens
    (1000, 6384, 128),     # wide tile (with its prefetches at 2 bits, PoT), ragged
])
def test_gemm_many_token_tiles_other_widths_and_groups(potq, bits, group, M, N, K):
    """The tiles above 64 tokens at the code widths and the group size the other tests leave out."""
    for is_int in (False, True):
        packed, S, Z = _gemv_inputs(3000 + M + bits + group, N, K, bits, is_int, group)
        X = workloads.activations(3100 + M, M, K)
        want = oracle.gemm(packed, S, Z, X, K, bits, group, nthreads=8)
        got = _run_gemm(potq, packed, S, Z, X, K, bits, group=group)
        e, nw, nfloor = rel_err(got, want, K)
        assert e <= REL_TOL, (is_int, e, nw, nfloor)


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("K", [32768, 53248, 76672])
def test_gemv_rows_beyond_64_kib_of_lds(potq, K, is_int):
    """x of long rows needs more LDS than a kernel gets by default (the limit is raised once per
    device); 76672 is the longest row the entry points accept."""
    bits, N = 3, 48
    packed = workloads.packed_codes(workloads.seed_of(9, K % 97, 0), N, K, bits)
    x = workloads.activations(workloads.seed_of(9, K % 97, 2), 1, K)
    tiled = potq.potq_repack(dev(packed), K, bits)
    if is_int:
        S, Z = workloads.int_scales_zeros(workloads.seed_of(9, K % 97, 3), N, K, bits, 128)
        got = host_bits(potq.int_gemv(tiled, dev(S), dev(Z), dev(x[0]), K, bits))
        got1 = host_bits(potq.int_gemm(tiled, dev(S), dev(Z), dev(x), K, bits))[0]
    else:
        S, Z = workloads.pot_scales(workloads.seed_of(9, K % 97, 1), N, K, 128), None
        got = host_bits(potq.pot_gemv(tiled, dev(S), dev(x[0]), K, bits))
        got1 = host_bits(potq.pot_gemm(tiled, dev(S), dev(x), K, bits))[0]
    want = oracle.gemm(packed, S, Z, x, K, bits, 128)[0]
    e, nw, nfloor = rel_err(got, want, K)
    assert e <= REL_TOL, (K, is_int, e, nw, nfloor)
    assert np.array_equal(got, got1)          # one token through the GEMM entry point is the same launch
    if is_int:
        ys = potq.int_gemv_batch([(tiled, dev(S), dev(Z)), (tiled, dev(S), dev(Z))],
                                 dev(x[0]), K, bits)
    else:
        ys = potq.pot_gemv_batch([(tiled, dev(S)), (tiled, dev(S))], dev(x[0]), K, bits)
    for y in ys:
        e, nw, nfloor = rel_err(host_bits(y), want, K)
        assert e <= REL_TOL, (K, is_int, e, nw, nfloor)
        if is_int or K > 32768:               # the multi-matrix launch shares the kernel body (PoT batches with
            assert np.array_equal(host_bits(y), got)   # rows up to 32768 run in the exponent form instead)
