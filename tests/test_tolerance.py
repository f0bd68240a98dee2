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


def test_outputs_below_the_normal_range_may_differ_by_one_quantum():
    """An output below 2^-14 is a multiple of the fp16 subnormal quantum 2^-24.  The fp64 oracle rounds the
    exact sum to that grid once; a kernel that accumulates in binary32 rounds a sum that differs from the
    exact one by far less than a quantum, so the two roundings agree or land on neighbouring multiples --
    never further apart.  One quantum is a relative error far above 2e-3 there (it is 2^-10 of the largest
    subnormal and 100 % of the smallest), which is why the GPU tests of tiny activations allow one quantum
    on top of the gate for such outputs, and nothing more."""
    bits, K, N, M = 3, 4096, 192, 4
    packed = workloads.packed_codes(9300, N, K, bits)
    S = workloads.pot_scales(9301, N, K, 128)
    X = (workloads.activations(9302, M, K).astype(np.float32) * np.float32(3e-7)).astype(np.float16)   # subnormal x
    want = oracle.gemm(packed, S, None, X, K, bits, 128, nthreads=4).view(np.float16).astype(np.float64)
    W = oracle.pot_dequant(packed, S, K, bits, 128, nthreads=4).view(np.float16).astype(np.float64)
    ideal = _fp32_chain(X.astype(np.float64), W).astype(np.float16).astype(np.float64)
    small = np.abs(want) < 2.0 ** -14
    assert small.mean() > 0.9                       # the case is what it is meant to be
    quantum = 2.0 ** -24
    diff = np.abs(ideal - want)
    assert diff[small].max() <= quantum             # neighbouring multiples at most
    # the plain gate would reject such a neighbour: the allowance is needed, and it is one quantum, not two
    rms = np.sqrt(np.mean(want * want))
    gate = REL_TOL * np.maximum(np.abs(want), rms * _floor_fraction(K))
    assert gate[small].max() < quantum
    # the allowance the GPU tests use: gate + one quantum below the normal range
    allowed = gate + np.where(small, quantum, 0.0)
    assert np.all(diff <= allowed)
    # two quanta off is outside it
    assert np.all((2 * quantum > allowed)[small])
