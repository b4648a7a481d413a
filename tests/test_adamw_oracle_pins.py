"""Pins of the AdamW oracle (the fallback for vector-valued parameters, Sec. 4.1): a library
implementation of the same published algorithm, closed forms, and planted mistakes."""
import numpy as np
import pytest
import torch

from oracle import adamw_oracle as ao
from oracle.adamw_oracle import AdamWHParams, AdamWOracle


def stream(shape, seed, K):
    r = np.random.default_rng(seed)
    return [r.standard_normal(shape) * 10.0 ** r.uniform(-4, 0) for _ in range(K)]


@pytest.mark.parametrize("hp", [AdamWHParams(), AdamWHParams(3e-2, 0.8, 0.999, 1e-6, 0.0),
                                AdamWHParams(1e-2, 0.0, 0.5, 1e-3, 0.5)])
def test_against_torch_adamw_in_float64(hp):
    shape, K = (5, 7), 8
    w0 = np.random.default_rng(1).standard_normal(shape)
    G = stream(shape, 2, K)
    p = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=hp.lr, betas=(hp.beta1, hp.beta2), eps=hp.eps, weight_decay=hp.weight_decay)
    o = AdamWOracle(shape)
    w = w0.copy()
    for k in range(K):
        p.grad = torch.tensor(G[k], dtype=torch.float64)
        opt.step()
        w = o.step(w, G[k], hp)
        np.testing.assert_allclose(w, p.detach().numpy(), rtol=1e-12, atol=1e-15)
    st = opt.state[p]
    np.testing.assert_allclose(o.m, st["exp_avg"].numpy(), rtol=1e-12, atol=1e-300)
    np.testing.assert_allclose(o.v, st["exp_avg_sq"].numpy(), rtol=1e-12, atol=1e-300)
    assert o.t == K


def test_first_step_and_constant_gradient_closed_forms():
    hp = AdamWHParams(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    g = np.array([[2.0, -0.5, 1e-3, 0.0, -7.0]])
    w0 = np.array([[1.0, -2.0, 0.5, 3.0, 0.0]])
    o = AdamWOracle(g.shape)
    w = o.step(w0, g, hp)
    # t = 1: mhat = g, vhat = g^2 whatever the betas
    want = w0 - hp.lr * (g / (np.abs(g) + hp.eps) + hp.weight_decay * w0)
    np.testing.assert_allclose(w, want, rtol=1e-14, atol=1e-18)
    # a constant gradient keeps mhat = g and vhat = g^2 at every step:
    # w_t = (1 - eta lambda)^t w_0 - eta s (1 - (1 - eta lambda)^t) / (eta lambda),  s = g / (|g| + eps)
    for t in range(2, 12):
        w = o.step(w, g, hp)
        np.testing.assert_allclose(o.m, g * (1 - hp.beta1 ** t), rtol=1e-13)
        np.testing.assert_allclose(o.v, g * g * (1 - hp.beta2 ** t), rtol=1e-13)
    q = 1.0 - hp.lr * hp.weight_decay
    s = g / (np.abs(g) + hp.eps)
    want = q ** 11 * w0 - hp.lr * s * (1 - q ** 11) / (hp.lr * hp.weight_decay)
    np.testing.assert_allclose(w, want, rtol=1e-11, atol=1e-15)
    # zero gradient: only the decay acts, and 0 / (0 + eps) is 0
    assert w[0, 3] == pytest.approx(3.0 * q ** 11, rel=1e-13)


def _pins_pass():
    try:
        test_against_torch_adamw_in_float64(AdamWHParams())
        test_first_step_and_constant_gradient_closed_forms()
    except AssertionError:
        return False
    return True


def test_planted_mistakes_are_caught(monkeypatch):
    assert _pins_pass()

    def no_bias_correction(self, w, g, hp):
        w = np.asarray(w, dtype=np.float64); g = np.asarray(g, dtype=np.float64)
        self.t += 1
        self.m = hp.beta1 * self.m + (1 - hp.beta1) * g
        self.v = hp.beta2 * self.v + (1 - hp.beta2) * g * g
        return w - hp.lr * (self.m / (np.sqrt(self.v) + hp.eps) + hp.weight_decay * w)

    def coupled_decay(self, w, g, hp):
        w = np.asarray(w, dtype=np.float64); g = np.asarray(g, dtype=np.float64) + hp.weight_decay * w
        self.t += 1
        self.m = hp.beta1 * self.m + (1 - hp.beta1) * g
        self.v = hp.beta2 * self.v + (1 - hp.beta2) * g * g
        mhat = self.m / (1 - hp.beta1 ** self.t); vhat = self.v / (1 - hp.beta2 ** self.t)
        return w - hp.lr * mhat / (np.sqrt(vhat) + hp.eps)

    def eps_inside_root(self, w, g, hp):
        w = np.asarray(w, dtype=np.float64); g = np.asarray(g, dtype=np.float64)
        self.t += 1
        self.m = hp.beta1 * self.m + (1 - hp.beta1) * g
        self.v = hp.beta2 * self.v + (1 - hp.beta2) * g * g
        mhat = self.m / (1 - hp.beta1 ** self.t); vhat = self.v / (1 - hp.beta2 ** self.t)
        return w - hp.lr * (mhat / np.sqrt(vhat + hp.eps) + hp.weight_decay * w)

    def swapped_betas(self, w, g, hp):
        w = np.asarray(w, dtype=np.float64); g = np.asarray(g, dtype=np.float64)
        self.t += 1
        self.m = hp.beta2 * self.m + (1 - hp.beta2) * g
        self.v = hp.beta1 * self.v + (1 - hp.beta1) * g * g
        mhat = self.m / (1 - hp.beta2 ** self.t); vhat = self.v / (1 - hp.beta1 ** self.t)
        return w - hp.lr * (mhat / (np.sqrt(vhat) + hp.eps) + hp.weight_decay * w)

    for bad in (no_bias_correction, coupled_decay, eps_inside_root, swapped_betas):
        monkeypatch.setattr(AdamWOracle, "step", bad)
        assert not _pins_pass(), bad.__name__
    monkeypatch.undo()
    assert _pins_pass()
