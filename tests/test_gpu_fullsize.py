"""GPU parity at the full sizes of the benchmark workloads, through the same
entry points and launch configurations bench.py times.  Where the oracle can
afford it the whole output is compared; for the 70B / 13B sizes a random sample
of weight rows is compared against the oracle and properties that hold for any
in-domain input are checked on the whole output (on the GPU, with integer ops)."""
import numpy as np
import pytest
import torch

import oracle
import workloads
from gpu_util import REL_TOL, dev, host_bits, rel_err

pytestmark = pytest.mark.gpu
G = workloads.GROUP


@pytest.fixture(scope="module")
def potq():
    import paper_2507_11959_amd as p
    return p


def _threads():
    import os
    return min(16, len(os.sched_getaffinity(0)))


def _invariants(out: torch.Tensor, scales: torch.Tensor, codes_sampled_ok: bool, bits: int):
    """Low 10 bits = the group's scale's, exponent field moved by 0..qmax, computed on the GPU."""
    qmax = 2 ** (bits - 1) - 1
    o = out.view(torch.int16).to(torch.int32) & 0xFFFF
    s = scales.view(torch.int16).to(torch.int32) & 0xFFFF
    s = s.repeat_interleave(G, dim=1)
    assert bool(((o & 0x3FF) == (s & 0x3FF)).all())
    d = ((o >> 10) & 31) - ((s >> 10) & 31)
    assert int(d.min()) >= 0 and int(d.max()) <= qmax
    # with uniform random codes every level and both signs occur
    assert int(d.max()) == qmax and int((o >> 15).max()) == 1 and int((o >> 15).min()) == 0


def test_config0_single_4096_3bit_dequant_full(potq):
    N, K, bits = 4096, 4096, 3
    packed, scales = workloads.pot_matrix(0, 0, N, K, bits, G)
    want = oracle.pot_dequant(packed, scales, K, bits, G, nthreads=_threads())
    got = host_bits(potq.pot_dequant(dev(packed), dev(scales), K, bits, G))
    assert np.array_equal(got, want)


@pytest.mark.parametrize("is_int", [False, True])
def test_config1_llama7b_layer_2bit_batch_full(potq, is_int):
    bits = 2
    mats, wants = [], []
    for i, (name, N, K) in enumerate(workloads.LLAMA2_7B_LAYER):
        packed = workloads.packed_codes(workloads.seed_of(1, i, 0), N, K, bits)
        out = torch.empty((N, K), dtype=torch.float16, device="cuda:0")
        if is_int:
            S, Z = workloads.int_scales_zeros(workloads.seed_of(1, i, 3), N, K, bits, G)
            mats.append((dev(packed), dev(S), dev(Z), out, K))
            wants.append((packed, S, Z))
        else:
            S = workloads.pot_scales(workloads.seed_of(1, i, 1), N, K, G)
            mats.append((dev(packed), dev(S), out, K))
            wants.append((packed, S, None))
    if is_int:
        potq.int_dequant_batch(mats, bits, G)
    else:
        potq.pot_dequant_batch(mats, bits, G)
    for m, (packed, S, Z), (name, N, K) in zip(mats, wants, workloads.LLAMA2_7B_LAYER):
        if is_int:
            want = oracle.int_dequant(packed, S, Z, K, bits, G, nthreads=_threads())
        else:
            want = oracle.pot_dequant(packed, S, K, bits, G, nthreads=_threads())
        assert np.array_equal(host_bits(m[-2]), want), name


@pytest.mark.parametrize("bits", [2, 3])
def test_config3_llama70b_layer_dequant_sampled_and_invariants(potq, bits):
    rng = np.random.default_rng(70 + bits)
    mats, keep = [], []
    for i, (name, N, K) in enumerate(workloads.LLAMA2_70B_LAYER):
        packed, scales = workloads.pot_matrix(3, i, N, K, bits, G)
        out = torch.empty((N, K), dtype=torch.float16, device="cuda:0")
        d_scales = dev(scales)
        mats.append((dev(packed), d_scales, out, K))
        keep.append((name, N, K, packed, scales))
    potq.pot_dequant_batch(mats, bits, G)
    for (name, N, K, packed, scales), m in zip(keep, mats):
        rows = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, 96)]))
        want = oracle.pot_dequant(packed[rows], scales[rows], K, bits, G, nthreads=_threads())
        got = host_bits(m[2][torch.from_numpy(rows).to("cuda:0")])
        assert np.array_equal(got, want), name
        _invariants(m[2], m[1], True, bits)


@pytest.mark.parametrize("is_int", [False, True])
def test_config2_gemv_3bit_7b_shapes_full(potq, is_int):
    bits = 3
    for i, (name, N, K) in enumerate(workloads.GEMV_7B_SHAPES):
        packed = workloads.packed_codes(workloads.seed_of(2, i, 0), N, K, bits)
        x = workloads.activations(workloads.seed_of(2, i, 2), 1, K)
        tiled = potq.potq_repack(dev(packed), K, bits)
        if is_int:
            S, Z = workloads.int_scales_zeros(workloads.seed_of(2, i, 3), N, K, bits, G)
            got = host_bits(potq.int_gemv(tiled, dev(S), dev(Z), dev(x[0]), K, bits))
        else:
            S, Z = workloads.pot_scales(workloads.seed_of(2, i, 1), N, K, G), None
            got = host_bits(potq.pot_gemv(tiled, dev(S), dev(x[0]), K, bits))
        want = oracle.gemm(packed, S, Z, x, K, bits, G, nthreads=_threads())[0]
        e, nw, nfloor = rel_err(got, want, K)
        assert e <= REL_TOL, (name, e, nw, nfloor)


@pytest.mark.parametrize("bits", [2, 3])
def test_config3_llama70b_gemv_full(potq, bits):
    for i, (name, N, K) in enumerate(workloads.LLAMA2_70B_LAYER):
        if i in (1, 3, 5):      # o, v, up repeat the shapes of q, k, gate
            continue
        packed, S = workloads.pot_matrix(3, i, N, K, bits, G)
        x = workloads.activations(workloads.seed_of(3, i, 2), 1, K)
        tiled = potq.potq_repack(dev(packed), K, bits)
        got = host_bits(potq.pot_gemv(tiled, dev(S), dev(x[0]), K, bits))
        want = oracle.gemm(packed, S, None, x, K, bits, G, nthreads=_threads())[0]
        e, nw, nfloor = rel_err(got, want, K)
        assert e <= REL_TOL, (name, e, nw, nfloor)


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("M", workloads.GEMM_TOKENS)
def test_config4_gemm_3bit_13b_shapes_sampled_rows(potq, M, is_int):
    bits = 3
    rng = np.random.default_rng(13 + M)
    for i, (name, N, K) in enumerate(workloads.GEMM_13B_SHAPES):
        packed = workloads.packed_codes(workloads.seed_of(4, i, 0), N, K, bits)
        X = workloads.activations(workloads.seed_of(4, i, 2) + M, M, K)
        tiled = potq.potq_repack(dev(packed), K, bits)
        if is_int:
            S, Z = workloads.int_scales_zeros(workloads.seed_of(4, i, 3), N, K, bits, G)
            Y = potq.int_gemm(tiled, dev(S), dev(Z), dev(X), K, bits, workspace=potq.gemm_workspace(M, N, K, bits))
        else:
            S, Z = workloads.pot_scales(workloads.seed_of(4, i, 1), N, K, G), None
            Y = potq.pot_gemm(tiled, dev(S), dev(X), K, bits, workspace=potq.gemm_workspace(M, N, K, bits))
        rows = np.unique(np.concatenate([[0, 15, 16, N - 1], rng.integers(0, N, 200)]))
        want = oracle.gemm(packed[rows], S[rows], None if Z is None else Z[rows], X, K, bits, G,
                           nthreads=_threads())
        got = host_bits(Y[:, torch.from_numpy(rows).to("cuda:0")].contiguous())
        e, nw, nfloor = rel_err(got, want, K)
        assert e <= REL_TOL, (name, M, e, nw, nfloor)
        assert bool(torch.isfinite(Y).all())


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("M,N,K", [
    (128, 5120, 5120),      # narrow tile, K split six ways
    (256, 8192, 8192),      # wide tile, K split four ways
    (512, 5120, 13824),     # wide tile, K split three ways
    (1000, 28672, 8192),    # wide tile, no split, ragged token tile
    (2048, 13824, 5120),    # tall tile, no split
])
def test_gemm_many_tokens_every_tile_and_split_sampled_rows(potq, M, N, K, is_int):
    """More than 64 tokens: the tile (wide, narrow, tall) and the number of K splits come from the
    dispatcher's cost model; one full-size case for each kind of plan, with the preferred workspace."""
    bits = 3
    rng = np.random.default_rng(90 + M)
    packed = workloads.packed_codes(workloads.seed_of(8, M % 7, 0), N, K, bits)
    X = workloads.activations(workloads.seed_of(8, M % 7, 2), M, K)
    tiled = potq.potq_repack(dev(packed), K, bits)
    ws = potq.gemm_workspace(M, N, K, bits)
    if is_int:
        S, Z = workloads.int_scales_zeros(workloads.seed_of(8, M % 7, 3), N, K, bits, G)
        Y = potq.int_gemm(tiled, dev(S), dev(Z), dev(X), K, bits, workspace=ws)
        again = potq.int_gemm(tiled, dev(S), dev(Z), dev(X), K, bits, workspace=ws)
    else:
        S, Z = workloads.pot_scales(workloads.seed_of(8, M % 7, 1), N, K, G), None
        Y = potq.pot_gemm(tiled, dev(S), dev(X), K, bits, workspace=ws)
        again = potq.pot_gemm(tiled, dev(S), dev(X), K, bits, workspace=ws)
    assert torch.equal(Y, again)                      # fixed summation order: bit-identical reruns
    del again
    rows = np.unique(np.concatenate([[0, 15, 16, 255, 256, 383, 384, N - 1], rng.integers(0, N, 100)]))
    want = oracle.gemm(packed[rows], S[rows], None if Z is None else Z[rows], X, K, bits, G, nthreads=_threads())
    got = host_bits(Y[:, torch.from_numpy(rows).to("cuda:0")].contiguous())
    e, nw, nfloor = rel_err(got, want, K)
    assert e <= REL_TOL, ((M, N, K), e, nw, nfloor)
    assert bool(torch.isfinite(Y).all())
    del tiled, Y, ws
    torch.cuda.empty_cache()


@pytest.mark.parametrize("is_int", [False, True])
@pytest.mark.parametrize("M", [24, 32, 64])
def test_gemm_few_row_tiles_large_matrices_sampled_rows(potq, M, is_int):
    """17 to 64 tokens on large matrices with N <= 8192 (four row tiles per wavefront; K split inside
    the workgroup for K <= 8192, over workgroups for longer rows)."""
    bits = 3
    rng = np.random.default_rng(70 + M)
    for i, (N, K) in enumerate([(8192, 8192), (6656, 6656), (8192, 28672), (6656, 17920)]):
        packed = workloads.packed_codes(workloads.seed_of(7, i, 0), N, K, bits)
        X = workloads.activations(workloads.seed_of(7, i, 2) + M, M, K)
        tiled = potq.potq_repack(dev(packed), K, bits)
        if is_int:
            S, Z = workloads.int_scales_zeros(workloads.seed_of(7, i, 3), N, K, bits, G)
            Y = potq.int_gemm(tiled, dev(S), dev(Z), dev(X), K, bits, workspace=potq.gemm_workspace(M, N, K, bits))
        else:
            S, Z = workloads.pot_scales(workloads.seed_of(7, i, 1), N, K, G), None
            Y = potq.pot_gemm(tiled, dev(S), dev(X), K, bits, workspace=potq.gemm_workspace(M, N, K, bits))
        rows = np.unique(np.concatenate([[0, 15, 16, 63, 64, N - 1], rng.integers(0, N, 120)]))
        want = oracle.gemm(packed[rows], S[rows], None if Z is None else Z[rows], X, K, bits, G,
                           nthreads=_threads())
        got = host_bits(Y[:, torch.from_numpy(rows).to("cuda:0")].contiguous())
        e, nw, nfloor = rel_err(got, want, K)
        assert e <= REL_TOL, ((N, K), M, e, nw, nfloor)
        assert bool(torch.isfinite(Y).all())
        del tiled, Y
    torch.cuda.empty_cache()


@pytest.mark.parametrize("N,K,bits,group,is_int", [
    (65552, 4096, 3, 128, True),      # vocabulary-sized: a resident grid of workgroups walks the row tiles
    (65552, 4096, 4, 64, False),      # 4-bit PoT, group size 64
    (16400, 16384, 2, 128, True),     # long rows (x fetched by the lanes of result column 0 only), ragged tile count
])
def test_gemv_vocabulary_sized_matrices_sampled_rows(potq, N, K, bits, group, is_int):
    rng = np.random.default_rng(N + bits)
    packed = workloads.packed_codes(workloads.seed_of(8, bits, 0), N, K, bits)
    x = workloads.activations(workloads.seed_of(8, bits, 2), 1, K)
    tiled = potq.potq_repack(dev(packed), K, bits)
    if is_int:
        S, Z = workloads.int_scales_zeros(workloads.seed_of(8, bits, 3), N, K, bits, group)
        y = potq.int_gemv(tiled, dev(S), dev(Z), dev(x[0]), K, bits, group)
    else:
        S, Z = workloads.pot_scales(workloads.seed_of(8, bits, 1), N, K, group), None
        y = potq.pot_gemv(tiled, dev(S), dev(x[0]), K, bits, group)
    rows = np.unique(np.concatenate([[0, 15, 16, N - 17, N - 1], rng.integers(0, N, 2000)]))
    want = oracle.gemm(packed[rows], S[rows], None if Z is None else Z[rows], x, K, bits, group,
                       nthreads=_threads())[0]
    e, nw, nfloor = rel_err(host_bits(y[torch.from_numpy(rows).to("cuda:0")]), want, K)
    assert e <= REL_TOL, (N, K, bits, group, is_int, e, nw, nfloor)
    assert bool(torch.isfinite(y).all())


@pytest.mark.parametrize("N,K,bits", [(32000, 4096, 3), (128256, 4096, 3), (128256, 8192, 3), (128256, 8192, 2)])
def test_pot_gemv_vocabulary_projections_exponent_form_sampled_rows(potq, N, K, bits):
    """The vocabulary projections bench.py times (PoT, exponent form: a grid of resident workgroups, each
    walking every grid-th pair of row tiles).  Sampled against the oracle: every row of the tile pairs on
    either side of each multiple of the grid size (where a workgroup moves on to its next pair, for grids of
    250 to 256 workgroups), of the first and the last pairs (the last one is the ragged end), and 1500 random rows."""
    assert potq.potq_gemv_exponent_form(N, K, bits)
    rng = np.random.default_rng(N + K + bits)
    packed, S = workloads.pot_matrix(8, 10 + bits, N, K, bits, G)
    x = workloads.activations(workloads.seed_of(8, 10 + bits, 2), 1, K)
    y = potq.pot_gemv(potq.potq_repack(dev(packed), K, bits), dev(S), dev(x[0]), K, bits, G)
    pairs = (N // 16 + 1) // 2                                    # tile pairs (32 rows each)
    edge = {0, 1, pairs - 2, pairs - 1}
    for grid in range(250, 257):
        for k in range(1, 4):
            edge.update({k * grid - 1, k * grid, k * grid + 1})
        edge.update({(pairs // grid) * grid - 1, (pairs // grid) * grid})
    edge_rows = np.concatenate([np.arange(32 * p, min(32 * p + 32, N)) for p in sorted(edge) if 0 <= p < pairs])
    rows = np.unique(np.concatenate([edge_rows, rng.integers(0, N, 1500)]))
    want = oracle.gemm(packed[rows], S[rows], None, x, K, bits, G, nthreads=_threads())[0]
    e, nw, nfloor = rel_err(host_bits(y[torch.from_numpy(rows).to("cuda:0")]), want, K)
    assert e <= REL_TOL, (N, K, bits, e, nw, nfloor)
    assert bool(torch.isfinite(y).all())


@pytest.mark.parametrize("bits", [2, 3])
def test_second_workload_llama30b_layer(potq, bits):
    """LLaMA-30B-shaped layer: batched dequant (sampled rows + invariants) and the q/k/v and gate/up
    projections as shared-activation GEMV batches (whole outputs)."""
    rng = np.random.default_rng(30 + bits)
    layer = workloads.LLAMA_30B_LAYER
    host, mats = [], []
    for i, (name, N, K) in enumerate(layer):
        packed, scales = workloads.pot_matrix(5, i, N, K, bits, G)
        host.append((packed, scales))
        mats.append((dev(packed), dev(scales), torch.empty((N, K), dtype=torch.float16, device="cuda:0"), K))
    potq.pot_dequant_batch(mats, bits, G)
    for (name, N, K), (packed, scales), m in zip(layer, host, mats):
        rows = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, 64)]))
        want = oracle.pot_dequant(packed[rows], scales[rows], K, bits, G, nthreads=_threads())
        assert np.array_equal(host_bits(m[2][torch.from_numpy(rows).to("cuda:0")]), want), name
        _invariants(m[2], m[1], True, bits)
    del mats
    torch.cuda.empty_cache()
    for idxs in ([0, 1, 2], [4, 5]):                 # q, k, v share x; gate, up share x
        K = layer[idxs[0]][2]
        x = workloads.activations(workloads.seed_of(5, idxs[0], 2), 1, K)
        batch = [(potq.potq_repack(dev(host[i][0]), K, bits), dev(host[i][1])) for i in idxs]
        ys = potq.pot_gemv_batch(batch, dev(x[0]), K, bits)
        for i, y in zip(idxs, ys):
            want = oracle.gemm(host[i][0], host[i][1], None, x, K, bits, G, nthreads=_threads())[0]
            e, nw, nfloor = rel_err(host_bits(y), want, K)
            assert e <= REL_TOL, (layer[i][0], e, nw, nfloor)


@pytest.mark.parametrize("bits", [2, 3])
def test_dequant_output_beyond_four_gibibytes(potq, bits):
    # 36864 x 65536 = 2.4 G weights: element indices pass 2^31 and output byte offsets pass 2^32, so any
    # 32-bit index arithmetic in the kernel or its launch would show here.  Sampled rows (first, last, around the
    # 2^31-element and 2^32-byte marks) against the oracle; codes are random bytes drawn on the device.
    N, K = 36864, 65536
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(77 + bits)
    codes = torch.randint(0, 256, (N, K * bits // 8), dtype=torch.uint8, device="cuda:0", generator=gen)
    scales_h = workloads.pot_scales(workloads.seed_of(9, bits, 1), N, K, G)
    scales = dev(scales_h)
    out = potq.pot_dequant(codes, scales, K, bits, G)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 1, N - 2, N - 1], [32766, 32767, 32768, 32769],      # 2^31 elements, 2^32 bytes
                                     [16383, 16384], np.random.default_rng(bits).integers(0, N, 24)]))
    idx = torch.from_numpy(rows).to("cuda:0")
    want = oracle.pot_dequant(codes[idx].cpu().numpy(), scales_h[rows], K, bits, G, nthreads=_threads())
    assert np.array_equal(host_bits(out[idx]), want)
    # every row obeys the format invariants (checked on the GPU in slices to bound memory)
    for r0 in range(0, N, 4096):
        _invariants(out[r0:r0 + 4096], scales[r0:r0 + 4096], True, bits)
