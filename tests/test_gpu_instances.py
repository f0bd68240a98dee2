"""One case for every kernel instance the dispatchers can reach that the other GPU tests leave out.

The fused kernels are templates over code width, PoT / uniform, group size and launch shape; the
tests of behaviour (test_gpu_parity, test_gpu_fullsize, ...) mostly run at 3 bits and group 128.
Register allocation, spills and scheduling differ per instance, so every instance a caller can
reach gets a comparison with the oracle here: small shapes where the dispatch allows it, sampled
rows of large matrices (codes drawn on the device) where an instance only serves large ones."""
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


def _matrix(seed, N, K, bits, group, is_int):
    packed = workloads.packed_codes(seed, N, K, bits)
    if is_int:
        S, Z = workloads.int_scales_zeros(seed + 3, N, K, bits, group)
    else:
        S, Z = workloads.pot_scales(seed + 1, N, K, group), None
    return packed, S, Z


def _device_matrix(seed, N, K, bits, group, is_int):
    """A large matrix whose codes are drawn on the device: (tiled codes, canonical codes, S, Z)."""
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(seed)
    canonical = torch.randint(0, 256, (N, K * bits // 8), dtype=torch.uint8, device="cuda:0", generator=gen)
    if is_int:
        S, Z = workloads.int_scales_zeros(seed + 3, N, K, bits, group)
    else:
        S, Z = workloads.pot_scales(seed + 1, N, K, group), None
    return canonical, S, Z


def _sampled_rows(N, seed, count=24):
    rng = np.random.default_rng(seed)
    return np.unique(np.concatenate([[0, 15, 16, N - 17, N - 1], rng.integers(0, N, count)]))


def _check_rows(Y, rows, canonical, S, Z, X, K, bits, group, tag):
    """Y: device result (N,) or (M, N); compares the sampled rows with the oracle."""
    idx = torch.from_numpy(rows).to("cuda:0")
    packed = canonical[idx].cpu().numpy()
    want = oracle.gemm(packed, S[rows], None if Z is None else Z[rows], X, K, bits, group, nthreads=8)
    got = host_bits(Y[idx] if Y.dim() == 1 else Y[:, idx].contiguous())
    if Y.dim() == 1:
        want = want[0]
    e, nw, nfloor = rel_err(got, want, K)
    assert e <= REL_TOL, (tag, e, nw, nfloor)


# ---------------------------------------------------------------------------
# GEMV, one workgroup per tile: wavefronts per tile by row length (1, 2, 4, 8) and the fetch of x
# by column 0 only for long rows; single launch and shared-activation batch launch.
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("K", [384, 1024, 2048, 4096, 8320, 36864])
def test_gemv_and_batch_every_row_length_class(potq, K, bits, group, is_int):
    x = workloads.activations(7000 + K, 1, K)
    rows = [48, 16, 80]
    mats = [_matrix(7100 + 10 * i + bits + K, N, K, bits, group, is_int) for i, N in enumerate(rows)]
    tiled = [potq.potq_repack(dev(p), K, bits) for p, _, _ in mats]
    if is_int:
        ys = potq.int_gemv_batch([(t, dev(S), dev(Z)) for t, (_, S, Z) in zip(tiled, mats)], dev(x[0]), K, bits, group)
        single = potq.int_gemv(tiled[0], dev(mats[0][1]), dev(mats[0][2]), dev(x[0]), K, bits, group)
    else:
        ys = potq.pot_gemv_batch([(t, dev(S)) for t, (_, S, _) in zip(tiled, mats)], dev(x[0]), K, bits, group)
        single = potq.pot_gemv(tiled[0], dev(mats[0][1]), dev(x[0]), K, bits, group)
    for (packed, S, Z), y in zip(mats, ys):
        want = oracle.gemm(packed, S, Z, x, K, bits, group)[0]
        e, nw, nfloor = rel_err(host_bits(y), want, K)
        assert e <= REL_TOL, (e, nw, nfloor)
    # 2- and 3-bit PoT batches with 4096 <= K <= 32768 run in the exponent form, the small single
    # matrix in the fp16 form; everywhere else both launches do the same arithmetic in the same order
    if is_int or bits == 4 or K < 4096 or K > 32768:
        assert np.array_equal(host_bits(single), host_bits(ys[0]))


# Two to four tokens through the GEMV kernel (one activation vector per result column).
@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("M", [2, 4])
def test_gemm_two_to_four_tokens_other_widths(potq, M, bits, is_int):
    N, K = 48, 4096                                    # rows of at least 32 groups take this kernel
    packed, S, Z = _matrix(7300 + M + bits, N, K, bits, 128, is_int)
    X = workloads.activations(7310 + M, M, K)
    tiled = potq.potq_repack(dev(packed), K, bits)
    Y = potq.int_gemm(tiled, dev(S), dev(Z), dev(X), K, bits) if is_int else potq.pot_gemm(tiled, dev(S), dev(X), K, bits)
    e, nw, nfloor = rel_err(host_bits(Y), oracle.gemm(packed, S, Z, X, K, bits, 128), K)
    assert e <= REL_TOL, (e, nw, nfloor)


# Few-token GEMM on a tall matrix (sixteen wavefronts per workgroup).
@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_gemm_few_tokens_tall_matrix(potq, bits, group, is_int):
    M, N, K = 13, 12304, 384
    packed, S, Z = _matrix(7400 + bits + group, N, K, bits, group, is_int)
    X = workloads.activations(7410 + bits, M, K)
    tiled = potq.potq_repack(dev(packed), K, bits)
    if is_int:
        Y = potq.int_gemm(tiled, dev(S), dev(Z), dev(X), K, bits, group)
    else:
        Y = potq.pot_gemm(tiled, dev(S), dev(X), K, bits, group)
    e, nw, nfloor = rel_err(host_bits(Y), oracle.gemm(packed, S, Z, X, K, bits, group, nthreads=8), K)
    assert e <= REL_TOL, (e, nw, nfloor)


# The tiled GEMM's configurations for 17 to 64 tokens and the narrow tile above, at 2 and 4 bits
# (3 bits: test_gemm_every_dispatch_configuration; the wide and tall tiles at 2 and 4 bits:
# test_gemm_many_token_tiles_other_widths_and_groups).
@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("M,N,K", [
    (24, 80, 1280),        # K split inside the workgroup, two row tiles per wavefront
    (24, 32, 11008),       # long rows: one row tile per wavefront, K split over workgroups
    (30, 8208, 256),       # tall matrix
    (48, 8208, 384),
    (64, 48, 9216),
    (100, 16640, 128),     # narrow tile
])
def test_gemm_tiled_configurations_other_widths(potq, M, N, K, bits, is_int):
    packed, S, Z = _matrix(7500 + M + N + bits, N, K, bits, 128, is_int)
    X = workloads.activations(7510 + M, M, K)
    want = oracle.gemm(packed, S, Z, X, K, bits, 128, nthreads=8)
    tiled = potq.potq_repack(dev(packed), K, bits)
    for ws in (potq.gemm_workspace(M, N, K, bits), None):
        if is_int:
            Y = potq.int_gemm(tiled, dev(S), dev(Z), dev(X), K, bits, workspace=ws)
        else:
            Y = potq.pot_gemm(tiled, dev(S), dev(X), K, bits, workspace=ws)
        e, nw, nfloor = rel_err(host_bits(Y), want, K)
        assert e <= REL_TOL, (ws is not None, e, nw, nfloor)


# Four row tiles per wavefront (large matrices with at most 8192 rows, 17 to 64 tokens): K split
# inside the workgroup for K <= 8192, over workgroups for longer rows.
@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("M,N,K", [(32, 8192, 8192), (64, 8192, 8192), (32, 4096, 28672), (64, 4096, 28672)])
def test_gemm_four_row_tiles_other_widths(potq, M, N, K, bits, is_int):
    canonical, S, Z = _device_matrix(7600 + M + bits + K, N, K, bits, 128, is_int)
    tiled = potq.potq_repack(canonical, K, bits)
    X = workloads.activations(7610 + M, M, K)
    ws = potq.gemm_workspace(M, N, K, bits)
    if is_int:
        Y = potq.int_gemm(tiled, dev(S), dev(Z), dev(X), K, bits, workspace=ws)
    else:
        Y = potq.pot_gemm(tiled, dev(S), dev(X), K, bits, workspace=ws)
    _check_rows(Y, _sampled_rows(N, M + bits), canonical, S, Z, X, K, bits, 128, (M, N, K, bits, is_int))
    del tiled, canonical, Y, ws
    torch.cuda.empty_cache()


# ---------------------------------------------------------------------------
# The exponent form: group size 64 with many tile sets per workgroup, the shared-activation
# launch in its four shapes (eight or sixteen wavefronts by row length; one to three tile sets
# per workgroup), and the kernel for two to four vectors.
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("bits", [2, 3])
def test_exponent_form_group_64_many_tile_sets(potq, bits):
    N, K, group = 16912, 4096, 64
    canonical, S, _ = _device_matrix(7700 + bits, N, K, bits, group, False)
    assert potq.potq_gemv_exponent_form(N, K, bits)
    x = workloads.activations(7710 + bits, 1, K)
    y = potq.pot_gemv(potq.potq_repack(canonical, K, bits), dev(S), dev(x[0]), K, bits, group)
    _check_rows(y, _sampled_rows(N, bits), canonical, S, None, x, K, bits, group, (N, K, bits))


@pytest.mark.parametrize("group", [64, 128])
@pytest.mark.parametrize("bits", [2, 3])
@pytest.mark.parametrize("rows,K", [
    ((7680, 7680), 4096),      # eight wavefronts, at most two tile sets per workgroup
    ((12288, 12304), 4096),    # eight wavefronts, three tile sets per workgroup
    ((2048, 2064), 16384),     # sixteen wavefronts (the digits of x need more than 64 KB), one tile set
    ((8704, 8720), 16384),     # sixteen wavefronts, three tile sets per workgroup
])
def test_exponent_form_shared_activation_launch_shapes(potq, rows, K, bits, group):
    x = workloads.activations(7800 + K, 1, K)
    mats = [_device_matrix(7810 + 10 * i + bits + group, N, K, bits, group, False) for i, N in enumerate(rows)]
    tiled = [potq.potq_repack(c, K, bits) for c, _, _ in mats]
    ys = potq.pot_gemv_batch([(t, dev(S)) for t, (_, S, _) in zip(tiled, mats)], dev(x[0]), K, bits, group)
    for i, ((canonical, S, _), y) in enumerate(zip(mats, ys)):
        _check_rows(y, _sampled_rows(rows[i], i + bits), canonical, S, None, x, K, bits, group, (rows, K, bits, group, i))
    del mats, tiled, ys
    torch.cuda.empty_cache()


@pytest.mark.parametrize("M,N,K,bits", [
    (2, 16384, 4096, 2),       # two vectors, eight wavefronts
    (4, 16384, 4096, 2),       # four vectors, eight wavefronts
    (4, 16400, 4096, 3),
    (2, 8720, 16384, 3),       # two vectors, sixteen wavefronts
])
def test_exponent_form_two_to_four_vectors_other_instances(potq, M, N, K, bits):
    canonical, S, _ = _device_matrix(7900 + M + bits, N, K, bits, 128, False)
    X = workloads.activations(7910 + M, M, K)
    Y = potq.pot_gemm(potq.potq_repack(canonical, K, bits), dev(S), dev(X), K, bits)
    _check_rows(Y, _sampled_rows(N, M + bits), canonical, S, None, X, K, bits, 128, (M, N, K, bits))
    del canonical, Y
    torch.cuda.empty_cache()


# ---------------------------------------------------------------------------
# The tile-walking GEMV (at least 256 M weights; what the exponent form cannot serve: the
# uniform baseline, 4-bit codes, and 2-/3-bit PoT rows beyond 32768 columns).
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("N,K,bits,group,is_int", [
    (65552, 4096, 2, 128, True), (65552, 4096, 2, 64, True), (16400, 16384, 2, 64, True),
    (16400, 16384, 3, 128, True), (65552, 4096, 3, 64, True), (16400, 16384, 3, 64, True),
    (65552, 4096, 4, 128, True), (16400, 16384, 4, 128, True), (65552, 4096, 4, 64, True), (16400, 16384, 4, 64, True),
    (65552, 4096, 4, 128, False), (16400, 16384, 4, 128, False), (16400, 16384, 4, 64, False),
    (8208, 36864, 2, 128, False), (8208, 36864, 2, 64, False), (8208, 36864, 3, 128, False), (8208, 36864, 3, 64, False),
])
def test_tile_walking_gemv_other_instances(potq, N, K, bits, group, is_int):
    canonical, S, Z = _device_matrix(8000 + bits + group + K % 97, N, K, bits, group, is_int)
    tiled = potq.potq_repack(canonical, K, bits)
    x = workloads.activations(8010 + bits, 1, K)
    if is_int:
        y = potq.int_gemv(tiled, dev(S), dev(Z), dev(x[0]), K, bits, group)
    else:
        assert not potq.potq_gemv_exponent_form(N, K, bits)
        y = potq.pot_gemv(tiled, dev(S), dev(x[0]), K, bits, group)
    _check_rows(y, _sampled_rows(N, bits + group), canonical, S, Z, x, K, bits, group, (N, K, bits, group, is_int))
    del tiled, canonical, y
    torch.cuda.empty_cache()
