"""Pins for the oracle's actor loss (Section 5.1, eq. (1)) and its logit gradient
(Appendix A.4.2): automatic differentiation of the written-out loss in fp64, finite
differences, and the invariants the closed form must obey."""
import math

import numpy as np
import pytest
import torch

from paper_2410_14803_amd import synth


def _case(seed, N=3, A=2, V=11, masked=True):
    rng = np.random.default_rng(seed)
    R = N * A
    x = (rng.standard_normal((R, V)) * 2).astype(np.float32)
    bits = synth.f32_to_bf16_bits(x)
    tok = rng.integers(0, V, size=R).astype(np.int32)
    if masked:
        tok[1] = -1
    rho = np.exp(rng.standard_normal(N) * 0.5)
    target = rng.uniform(-1, 1, N)
    base = rng.uniform(-1, 1, N)
    pen = (rng.random(N) < 0.5).astype(float)
    return bits, tok, rho, target, base, pen


def _torch_loss(xd, tok, A, rho, target, base, pen, beta, lam, scale):
    """Eq. (1) written with library ops: log-softmax gather, Categorical entropy."""
    ls = torch.log_softmax(xd, dim=1)
    live = torch.from_numpy((tok >= 0) & (tok < xd.shape[1]))
    tk = torch.from_numpy(np.where((tok >= 0) & (tok < xd.shape[1]), tok, 0)).long()
    lp = ls[torch.arange(xd.shape[0]), tk] * live
    ent = torch.distributions.Categorical(logits=xd).entropy() * live
    N = xd.shape[0] // A
    step_lp = lp.reshape(N, A).sum(1)
    step_ent = ent.reshape(N, A).sum(1)
    coef = torch.from_numpy(rho * (target - base))
    return scale * (-(coef * step_lp) - beta * step_ent + lam * torch.from_numpy(pen)).sum()


@pytest.mark.parametrize("seed,beta", [(1, 0.0), (2, 0.01), (3, 0.7)])
def test_against_autograd(oracle, seed, beta):
    bits, tok, rho, target, base, pen = _case(seed)
    A, lam, scale = 2, 0.3, 1.0 / 3
    loss, grad = oracle.actor_loss_grad(bits, tok, A, rho, target, base, beta, scale, penalty=pen, lambda_pen=lam)
    xd = torch.from_numpy(synth.bf16_bits_to_f64(bits)).requires_grad_(True)
    L = _torch_loss(xd, tok, A, rho, target, base, pen, beta, lam, scale)
    L.backward()
    assert loss == pytest.approx(float(L.detach()), rel=1e-12, abs=1e-13)
    np.testing.assert_allclose(grad, xd.grad.numpy(), rtol=1e-10, atol=1e-13)
    assert np.all(grad[1] == 0)            # the padding row has no gradient


def test_finite_differences_of_the_oracle_loss(oracle):
    # central differences on exactly representable perturbations of the bf16 logits
    bits, tok, rho, target, base, pen = _case(4, masked=False)
    x = synth.bf16_bits_to_f64(bits)
    x = np.round(x * 8) / 8                     # multiples of 1/8: +-1/8 stays exact in bf16 here
    bits = synth.f32_to_bf16_bits(x.astype(np.float32))
    assert np.array_equal(synth.bf16_bits_to_f64(bits), x)
    beta, scale = 0.2, 0.5
    _, grad = oracle.actor_loss_grad(bits, tok, 2, rho, target, base, beta, scale)
    h = 0.125
    for (r, v) in [(0, 0), (2, 5), (5, int(tok[5])), (3, 10)]:
        xp, xm = x.copy(), x.copy()
        xp[r, v] += h; xm[r, v] -= h
        lp, _ = oracle.actor_loss_grad(synth.f32_to_bf16_bits(xp.astype(np.float32)), tok, 2, rho, target, base,
                                       beta, scale, want_grad=False)
        lm, _ = oracle.actor_loss_grad(synth.f32_to_bf16_bits(xm.astype(np.float32)), tok, 2, rho, target, base,
                                       beta, scale, want_grad=False)
        assert (lp - lm) / (2 * h) == pytest.approx(grad[r, v], rel=2e-2, abs=1e-4)   # O(h^2) truncation


def test_invariants(oracle):
    bits, tok, rho, target, base, pen = _case(5, N=4, A=3, V=37, masked=False)
    loss, grad = oracle.actor_loss_grad(bits, tok, 3, rho, target, base, 0.3, 1.0)
    # softmax is shift invariant, so every row of the gradient sums to zero
    np.testing.assert_allclose(grad.sum(1), 0.0, atol=1e-13)
    # beta = 0: -coef * (onehot - p)
    _, g0 = oracle.actor_loss_grad(bits, tok, 3, rho, target, base, 0.0, 1.0)
    x = synth.bf16_bits_to_f64(bits)
    p = np.exp(x - x.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
    coef = np.repeat(rho * (target - base), 3)
    onehot = np.zeros_like(p); onehot[np.arange(len(tok)), tok] = 1
    np.testing.assert_allclose(g0, -coef[:, None] * (onehot - p), rtol=1e-11, atol=1e-14)
    # linear in scale; the penalty moves the loss only
    l2, g2 = oracle.actor_loss_grad(bits, tok, 3, rho, target, base, 0.3, 2.0)
    np.testing.assert_allclose(g2, 2 * grad, rtol=1e-14)
    assert l2 == pytest.approx(2 * loss, rel=1e-14)
    l3, g3 = oracle.actor_loss_grad(bits, tok, 3, rho, target, base, 0.3, 1.0, penalty=pen, lambda_pen=0.5)
    np.testing.assert_array_equal(g3, grad)
    assert l3 - loss == pytest.approx(0.5 * pen.sum(), rel=1e-12)


def test_uniform_logits_have_no_entropy_gradient(oracle):
    V = 50
    bits = synth.f32_to_bf16_bits(np.full((2, V), 1.25, np.float32))
    tok = np.array([3, 7], np.int32)
    loss, grad = oracle.actor_loss_grad(bits, tok, 1, [0.0, 0.0], [0.0, 0.0], [0.0, 0.0], 1.0, 1.0)
    np.testing.assert_allclose(grad, 0.0, atol=1e-15)        # entropy is at its maximum
    assert loss == pytest.approx(-2 * math.log(V), rel=1e-13)
