"""The tolerance of the fused kernels, checked on the CPU against the arithmetic it is derived from.

An ideal fp32 accumulation (exact 32-product steps, one rounding to binary32 per
step, one final rounding to fp16), simulated in numpy, must sit well inside the
gate against the fp64 oracle; a planted mistake of the size of one product must
fall outside it.  No GPU code is involved.
"""
import numpy as np
import pytest

import oracle
import workloads

REL_TOL = 2e-3


def _floor_fraction(K):
    # the same formula as tests/gpu_util.py (that module needs torch with a GPU build; this test does not)
    return max(2.0 ** -10, 8.0 * 2.0 ** -24 * (K / 32.0) ** 0.5 / REL_TOL)


def _err(y16, ref16, K):
    y = y16.astype(np.float64).ravel()
    r = ref16.astype(np.float64).ravel()
    rms = np.sqrt(np.mean(r * r))
    return (np.abs(y - r) / np.maximum(np.abs(r), rms * _floor_fraction(K))).max()


def _fp32_chain(X, W, step=32):
    acc = np.zeros((X.shape[0], W.shape[0]), np.float32)
    for k0 in range(0, X.shape[1], step):
        acc = (acc.astype(np.float64) + X[:, k0:k0 + step] @ W[:, k0:k0 + step].T).astype(np.float32)
    return acc


def test_formula_matches_the_gpu_helper():
    import ast
    import os
    src = open(os.path.join(os.path.dirname(__file__), "gpu_util.py")).read()
    fn = next(n for n in ast.parse(src).body if isinstance(n, ast.FunctionDef) and n.name == "floor_fraction")
    ns = {"REL_TOL": REL_TOL}
    exec(compile(ast.Module([fn], []), "gpu_util.floor_fraction", "exec"), ns)
    for K in (128, 1280, 4096, 11008, 28672):
        assert ns["floor_fraction"](K) == _floor_fraction(K)


@pytest.mark.parametrize("bits,K,seed", [(2, 4096, 1), (3, 11008, 2), (4, 11008, 3), (3, 28672, 4)])
def test_ideal_fp32_accumulation_is_inside_the_gate(bits, K, seed):
    N, M = 96, 8
    packed = workloads.packed_codes(9000 + seed, N, K, bits)
    S = workloads.pot_scales(9100 + seed, N, K, 128)
    X = workloads.activations(9200 + seed, M, K)
    want = oracle.gemm(packed, S, None, X, K, bits, 128, nthreads=4).view(np.float16)
    W = oracle.pot_dequant(packed, S, K, bits, 128, nthreads=4).view(np.float16).astype(np.float64)
    X64 = X.astype(np.float64)
    ideal = _fp32_chain(X64, W)
    assert _err(ideal.astype(np.float16), want, K) <= REL_TOL / 2
    # one product of typical size left out of every output: far outside
    broken = ideal.astype(np.float64) - np.outer(X64[:, 5], W[:, 5])
    assert _err(broken.astype(np.float16), want, K) > 10 * REL_TOL
    # fp16 accumulation would fail as well (the gate is not vacuous for precision mistakes)
    acc16 = np.zeros((M, N), np.float16)
    for k0 in range(0, K, 32):
        acc16 = (acc16.astype(np.float64) + X64[:, k0:k0 + 32] @ W[:, k0:k0 + 32].T).astype(np.float16)
    assert _err(acc16, want, K) > REL_TOL
