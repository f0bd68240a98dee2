"""Pins for the oracle's Step 2 op (Sec. 3.3): the printed formulas run through torch's autograd in
float64 with a straight-through round, and hand-derived closed forms."""
import numpy as np
import pytest
import torch

import oracle
import workloads


def _away_from_thresholds(W, Shat_up, qmax, margin=1e-3):
    """Nudge weights whose log2(|w|/S^) lies within `margin` of a half-integer (a rounding tie) or is zero."""
    W = W.astype(np.float64).copy()
    W[W == 0] = 1e-3
    for _ in range(4):
        v = np.log2(np.abs(W) / Shat_up)
        near = np.abs((v - 0.5) - np.rint(v - 0.5)) < margin
        W[near] *= 1.01
        W = W.astype(np.float16).astype(np.float64)
    v = np.log2(np.abs(W) / Shat_up)
    assert not np.any(np.abs((v - 0.5) - np.rint(v - 0.5)) < margin / 4)
    return W.astype(np.float16)


def _autograd(W, S, Gamma, dWq, qmax, group):
    Wt = torch.tensor(W.astype(np.float64))
    St = torch.tensor(S.astype(np.float64))
    G = torch.tensor(Gamma.astype(np.float64), requires_grad=True)
    Shat = (St * (1 + G)).repeat_interleave(group, dim=1)
    v = torch.log2(Wt.abs() / Shat)
    v_ste = v + (torch.round(v) - v).detach()               # round() with the identity as its derivative
    E = torch.clamp(v_ste, 0, qmax)
    Wq = Shat * torch.sign(Wt) * torch.pow(torch.tensor(2.0, dtype=torch.float64), E)
    (Wq * torch.tensor(dWq.astype(np.float64))).sum().backward()
    return Wq.detach().numpy(), G.grad.numpy()


@pytest.mark.parametrize("bits,group", [(2, 128), (3, 128), (3, 64), (4, 128)])
def test_against_autograd_of_the_printed_formulas(bits, group):
    qmax = 2 ** (bits - 1) - 1
    N, K = 5, 512
    rng = np.random.default_rng(10 * bits + group)
    W = workloads.weights_f16(77 + bits, N, K)
    _, S = oracle.pot_quantize(W, bits, group)              # realistic Step 1 scales
    S = S.view(np.float16)
    Gamma = rng.uniform(-0.2, 0.2, size=S.shape).astype(np.float32)
    Shat32 = S.astype(np.float32) * (np.float32(1) + Gamma)
    W = _away_from_thresholds(W, np.repeat(Shat32.astype(np.float64), group, axis=1), qmax)
    dWq = rng.standard_normal((N, K)).astype(np.float16)
    Wq_ref, dG_ref = _autograd(W, Shat32.astype(np.float64) / (1 + Gamma.astype(np.float64)), Gamma, dWq, qmax, group)
    Wq = oracle.fakequant_forward(W, S, Gamma, bits, group).view(np.float16)
    assert np.array_equal(Wq, Wq_ref.astype(np.float16))
    dG = oracle.fakequant_backward(W, S, Gamma, dWq, bits, group)
    # the reference's S differs from the fp16 S by the binary32 rounding of S^ only: scale it back
    ratio = S.astype(np.float64) / (Shat32.astype(np.float64) / (1 + Gamma.astype(np.float64)))
    assert np.allclose(dG, dG_ref * ratio, rtol=1e-6, atol=1e-9)
    assert np.abs(dG).max() > 0                              # the clamp is active somewhere: not a vacuous check
    # threads do not change the result
    assert np.array_equal(oracle.fakequant_backward(W, S, Gamma, dWq, bits, group, nthreads=4), dG)


def test_closed_forms():
    bits, group, qmax = 3, 128, 3
    S = np.full((3, 1), 0.25, np.float16)
    Gamma = np.array([[0.0], [0.5], [-0.5]], np.float32)     # S^ = 0.25, 0.375, 0.125
    g = np.ones((3, 128), np.float16)
    sign = np.where(np.arange(128) % 3 == 0, -1.0, 1.0)
    # (a) every weight inside the clamp's range: the two terms of dw~/dS^ cancel, gradient exactly 0
    W = (sign * 0.5).astype(np.float16)[None, :].repeat(3, 0)   # |w|/S^ = 2, 1.33, 4
    assert np.all(oracle.fakequant_backward(W, S, Gamma, g, bits, group) == 0)
    Wq = oracle.fakequant_forward(W, S, Gamma, bits, group).view(np.float16).astype(np.float64)
    assert np.array_equal(Wq, sign[None, :] * np.array([[0.5], [0.375], [0.5]]))   # E = 1, 0, 2
    # (b) every weight below range: w~ = sign * S^, dGamma = S * sum(g * sign)
    W = (sign * 0.01).astype(np.float16)[None, :].repeat(3, 0)
    assert np.array_equal(oracle.fakequant_forward(W, S, Gamma, bits, group).view(np.float16).astype(np.float64),
                          sign[None, :] * np.array([[0.25], [0.375], [0.125]]))
    assert np.all(oracle.fakequant_backward(W, S, Gamma, g, bits, group) == np.float32(0.25 * sign.sum()))
    # (c) every weight above range: E = qmax, dGamma = S * 2^qmax * sum(g * sign)
    W = (sign * 40.0).astype(np.float16)[None, :].repeat(3, 0)
    assert np.array_equal(oracle.fakequant_forward(W, S, Gamma, bits, group).view(np.float16).astype(np.float64),
                          sign[None, :] * 8 * np.array([[0.25], [0.375], [0.125]]))
    assert np.all(oracle.fakequant_backward(W, S, Gamma, g, bits, group) == np.float32(0.25 * 8 * sign.sum()))
    # (d) a zero weight: log2(0) = -inf is below range, sign(0) = +  ->  w~ = +S^ and it takes part in the gradient
    W = np.zeros((3, 128), np.float16)
    assert np.all(oracle.fakequant_forward(W, S, Gamma, bits, group).view(np.float16)[0] == np.float16(0.25))
    assert np.all(oracle.fakequant_backward(W, S, Gamma, g, bits, group) == np.float32(0.25 * 128))
    # (e) weights already on the grid of S are reproduced at Gamma = 0
    rng = np.random.default_rng(3)
    Wg = (rng.choice([-1.0, 1.0], (1, 128)) * 0.25 * 2.0 ** rng.integers(0, qmax + 1, (1, 128))).astype(np.float16)
    assert np.array_equal(oracle.fakequant_forward(Wg, S[:1], Gamma[:1], bits, group), Wg.view(np.uint16))


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_forward_at_gamma_zero_is_quantise_then_dequantise(bits):
    # with the Step 1 scale already rounded to fp16, Gamma = 0 must give decode(codes) of those codes re-derived
    # under that scale: compare with the printed formula in float64 away from ties
    qmax = 2 ** (bits - 1) - 1
    N, K, group = 4, 256, 128
    W = workloads.weights_f16(5 + bits, N, K)
    _, S = oracle.pot_quantize(W, bits, group)
    S = S.view(np.float16)
    Sup = np.repeat(S.astype(np.float64), group, axis=1)
    W = _away_from_thresholds(W, Sup, qmax)
    E = np.clip(np.rint(np.log2(np.abs(W.astype(np.float64)) / Sup)), 0, qmax)
    want = (np.sign(W.astype(np.float64)) * Sup * 2.0 ** E).astype(np.float16)
    got = oracle.fakequant_forward(W, S, np.zeros_like(S, dtype=np.float32), bits, group).view(np.float16)
    assert np.array_equal(got, want)
    # power-of-two equivariance: scaling W and S by 4 scales the result by 4
    got4 = oracle.fakequant_forward((W.astype(np.float32) * 4).astype(np.float16), (S.astype(np.float32) * 4)
                                    .astype(np.float16), np.zeros_like(S, dtype=np.float32), bits, group)
    assert np.array_equal(got4.view(np.float16), (got.astype(np.float32) * 4).astype(np.float16))
