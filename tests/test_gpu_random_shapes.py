"""Randomised (seeded) sweep of shapes, bit widths, group sizes and token counts through every entry point of the
hot path against the oracle: dequant and repack bit-exact, fused GEMV / GEMM within the stated tolerance."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import REL_TOL, dev, host_bits, rel_err

pytestmark = pytest.mark.gpu

TOKENS = [2, 3, 7, 15, 16, 17, 24, 31, 32, 33, 48, 63, 64, 65, 100, 128, 129, 200, 256, 300]


def _cases(seed, count):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        bits = int(rng.choice([2, 3, 4]))
        group = int(rng.choice([64, 128]))
        is_int = bool(rng.integers(0, 2))
        N = 16 * int(rng.integers(1, 40))
        K = 128 * int(rng.integers(1, 30))
        if rng.random() < 0.15:
            N = 16 * int(rng.integers(500, 700))       # tall: the many-row configurations
        if rng.random() < 0.15:
            K = 128 * int(rng.integers(60, 100))       # long rows: the long-K configurations
        M = int(rng.choice(TOKENS))
        if N * K * M > 1.5e9:
            M = 16                                      # keep the oracle's work bounded
        out.append((bits, group, is_int, N, K, M, int(rng.integers(0, 1 << 30))))
    return out


@pytest.mark.parametrize("chunk", range(6))
def test_random_shapes_against_the_oracle(chunk):
    import paper_2507_11959_amd as potq
    for bits, group, is_int, N, K, M, seed in _cases(20250711 + chunk, 10):
        tag = f"bits={bits} group={group} int={is_int} N={N} K={K} M={M} seed={seed}"
        packed = workloads.packed_codes(seed, N, K, bits)
        if is_int:
            S, Z = workloads.int_scales_zeros(seed + 1, N, K, bits, group)
            got = host_bits(potq.int_dequant(dev(packed), dev(S), dev(Z), K, bits, group))
            want = oracle.int_dequant(packed, S, Z, K, bits, group, nthreads=8)
        else:
            S, Z = workloads.pot_scales(seed + 1, N, K, group), None
            got = host_bits(potq.pot_dequant(dev(packed), dev(S), K, bits, group))
            want = oracle.pot_dequant(packed, S, K, bits, group, nthreads=8)
        assert np.array_equal(got, want), "dequant " + tag
        tiled = potq.potq_repack(dev(packed), K, bits)
        back = potq.potq_repack(tiled, K, bits, to_layout=potq.LAYOUT_CANONICAL)
        assert np.array_equal(back.cpu().numpy(), packed), "repack " + tag
        X = workloads.activations(seed + 2, M, K)
        wantY = oracle.gemm(packed, S, Z, X, K, bits, group, nthreads=8)
        if is_int:
            y = potq.int_gemv(tiled, dev(S), dev(Z), dev(X[0]), K, bits, group)
        else:
            y = potq.pot_gemv(tiled, dev(S), dev(X[0]), K, bits, group)
        e, _, _ = rel_err(host_bits(y), wantY[0], K)
        assert e <= REL_TOL, ("gemv", e, tag)
        for ws in (potq.gemm_workspace(M, N, K, bits), None):
            if is_int:
                Y = potq.int_gemm(tiled, dev(S), dev(Z), dev(X), K, bits, group, workspace=ws)
            else:
                Y = potq.pot_gemm(tiled, dev(S), dev(X), K, bits, group, workspace=ws)
            e, _, _ = rel_err(host_bits(Y), wantY, K)
            assert e <= REL_TOL, ("gemm", e, ws is not None, tag)
