"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds input recipes only: random packed code bytes, per-group
scales / zero-points with realistic values, Gaussian activations, and the
matrix shapes of the Llama-style decoder layers the workloads are quoted on.
It contains none of the de-quantisation arithmetic and imports neither the CPU
oracle nor the GPU package; both are fed from here.

Recipe (numpy Generator(PCG64(seed)), seed = 1_000_000*config + 1_000*matrix + kind):
  kind 0  packed codes: uniformly random bytes.  A dense stream of independent
          uniform b-bit codes is exactly a stream of independent uniform bits,
          so no packing step is involved.
  kind 1  PoT scales: s = fp16(max_{i<G} |w_i|), w_i ~ N(0, sigma^2), sigma = 0.02.
          The maximum is drawn directly from its distribution by inverse
          transform, max|w| = sigma * Phi^-1((1 + u^(1/G)) / 2), u ~ U(0,1), so a
          70B-sized layer needs one uniform per group instead of G Gaussians.
  kind 2  activations: fp16(N(0, 1)).
  kind 3  uniform-INT scale / zero-point: (max, min) of G draws of N(0, sigma^2)
          sampled jointly by inverse transform, S = fp16((max - min) / (2^b - 1)),
          Z = fp16(clip(round(min / S), -(2^b - 1), 0)) (an integer-valued fp16).
"""
from __future__ import annotations

import numpy as np
from scipy.special import ndtr, ndtri

SIGMA_W = 0.02
GROUP = 128

# (name, N = out features, K = in features)
LLAMA2_7B_LAYER = [("q", 4096, 4096), ("k", 4096, 4096), ("v", 4096, 4096), ("o", 4096, 4096),
                   ("gate", 11008, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
LLAMA2_70B_LAYER = [("q", 8192, 8192), ("o", 8192, 8192), ("k", 1024, 8192), ("v", 1024, 8192),
                    ("gate", 28672, 8192), ("up", 28672, 8192), ("down", 8192, 28672)]
# LLaMA-30B (hidden 6656, FFN 17920): the largest model the paper evaluates (Sec. 5.1)
LLAMA_30B_LAYER = [("q", 6656, 6656), ("k", 6656, 6656), ("v", 6656, 6656), ("o", 6656, 6656),
                   ("gate", 17920, 6656), ("up", 17920, 6656), ("down", 6656, 17920)]
GEMV_7B_SHAPES = [("attn", 4096, 4096), ("up", 11008, 4096), ("down", 4096, 11008)]
GEMM_13B_SHAPES = [("attn", 5120, 5120), ("up", 13824, 5120), ("down", 5120, 13824)]
GEMM_TOKENS = [16, 64, 256]

# index = position in the benchmark description's list of workloads
CONFIGS = {
    0: {"what": "single 4096x4096, 3-bit PoT dequant", "bits": [3], "shapes": [("w", 4096, 4096)]},
    1: {"what": "Llama-2-7B layer, 2-bit PoT + INT2 dequant", "bits": [2], "shapes": LLAMA2_7B_LAYER},
    2: {"what": "fused GEMV, 3-bit, 7B shapes", "bits": [3], "shapes": GEMV_7B_SHAPES},
    3: {"what": "Llama-2-70B layer, 2/3-bit dequant + GEMV", "bits": [2, 3], "shapes": LLAMA2_70B_LAYER},
    4: {"what": "fused GEMM, 3-bit, 13B shapes, M in 16/64/256", "bits": [3], "shapes": GEMM_13B_SHAPES},
    5: {"what": "second workload: LLaMA-30B layer, 2/3-bit dequant + GEMV", "bits": [2, 3], "shapes": LLAMA_30B_LAYER},
}


def seed_of(config: int, matrix: int, kind: int) -> int:
    return 1_000_000 * config + 1_000 * matrix + kind


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def packed_row_bytes(K: int, bits: int) -> int:
    assert (K * bits) % 8 == 0
    return K * bits // 8


def packed_codes(seed: int, N: int, K: int, bits: int) -> np.ndarray:
    """(N, K*bits/8) uint8 of uniformly random bytes."""
    rb = packed_row_bytes(K, bits)
    return _rng(seed).integers(0, 256, size=(N, rb), dtype=np.uint8)


def pot_scales(seed: int, N: int, K: int, group: int = GROUP, sigma: float = SIGMA_W) -> np.ndarray:
    """(N, K/group) float16, distributed as the max of `group` draws of |N(0, sigma^2)|."""
    u = _rng(seed).random(size=(N, K // group))
    m = sigma * ndtri(0.5 * (1.0 + u ** (1.0 / group)))
    return m.astype(np.float16)


def int_scales_zeros(seed: int, N: int, K: int, bits: int, group: int = GROUP, sigma: float = SIGMA_W):
    """(S, Z): two (N, K/group) float16 arrays for the uniform baseline."""
    r = _rng(seed)
    u = r.random(size=(N, K // group))
    v = r.random(size=(N, K // group))
    pmax = u ** (1.0 / group)                               # Phi(max / sigma)
    wmax = sigma * ndtri(pmax)
    wmin = sigma * ndtri(pmax * (1.0 - v ** (1.0 / (group - 1))))  # min of the others, given the max
    levels = float(2 ** bits - 1)
    S = ((wmax - wmin) / levels).astype(np.float16)
    Z = np.clip(np.rint(wmin / S.astype(np.float64)), -levels, 0.0).astype(np.float16)
    return S, Z


def activations(seed: int, M: int, K: int) -> np.ndarray:
    """(M, K) float16 ~ N(0, 1)."""
    return _rng(seed).standard_normal(size=(M, K)).astype(np.float16)


def weights_f16(seed: int, N: int, K: int, sigma: float = SIGMA_W) -> np.ndarray:
    """(N, K) float16 ~ N(0, sigma^2): stand-in for a trained weight matrix (input of the scale search)."""
    return (_rng(seed).standard_normal(size=(N, K), dtype=np.float32) * np.float32(sigma)).astype(np.float16)


def pot_matrix(config: int, matrix: int, N: int, K: int, bits: int, group: int = GROUP):
    """(packed codes, scales) of one PoT-quantised weight matrix."""
    return (packed_codes(seed_of(config, matrix, 0), N, K, bits),
            pot_scales(seed_of(config, matrix, 1), N, K, group))


def int_matrix(config: int, matrix: int, N: int, K: int, bits: int, group: int = GROUP):
    """(packed codes, S, Z) of one uniformly quantised weight matrix (same code bytes as the PoT one)."""
    S, Z = int_scales_zeros(seed_of(config, matrix, 3), N, K, bits, group)
    return packed_codes(seed_of(config, matrix, 0), N, K, bits), S, Z


def algorithmic_bytes_dequant(N: int, K: int, bits: int, group: int, with_zeros: bool = False) -> int:
    """HBM bytes a stand-alone dequant must move: codes + scales (+ zero-points) in, fp16 out."""
    per_group = 2 * (2 if with_zeros else 1)
    return N * K * bits // 8 + N * (K // group) * per_group + 2 * N * K


def algorithmic_bytes_gemm(M: int, N: int, K: int, bits: int, group: int, with_zeros: bool = False) -> int:
    """HBM bytes of a fused dequant + GEMV/GEMM: codes + scales (+ zeros) + X in, Y out."""
    per_group = 2 * (2 if with_zeros else 1)
    return N * K * bits // 8 + N * (K // group) * per_group + 2 * M * K + 2 * M * N
