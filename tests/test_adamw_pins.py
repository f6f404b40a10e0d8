"""Pins of the AdamW oracle against closed forms, a hand-worked sequence and torch's CPU implementation."""
import numpy as np
import pytest

from oracle import adamw_oracle as ao


def test_first_step_closed_form():
    # t = 1 from zero moments: mhat = g, vhat = g^2, so the update is -lr g / (|g| + eps) - lr wd w
    rng = np.random.default_rng(0)
    w, g = rng.normal(size=50), rng.normal(size=50)
    z = np.zeros(50)
    w1, m1, v1 = ao.adamw_step(w, g, z, z, 1, lr=0.01, eps=1e-8, weight_decay=0.1)
    np.testing.assert_allclose(w1, w - 0.01 * (g / (np.abs(g) + 1e-8) + 0.1 * w), rtol=1e-12, atol=0)
    np.testing.assert_allclose(m1, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v1, 0.001 * g * g, rtol=1e-9)


def test_zero_gradient_is_pure_decay():
    w, m, v = np.array([2.0, -3.0]), np.array([0.5, -0.25]), np.array([0.04, 0.09])
    g = np.zeros(2)
    w1, m1, v1 = ao.adamw_step(w, g, m, v, 7, lr=0.1, beta1=0.9, beta2=0.99, eps=1e-3, weight_decay=0.5)
    np.testing.assert_allclose(m1, 0.9 * m, rtol=1e-15)
    np.testing.assert_allclose(v1, 0.99 * v, rtol=1e-15)
    mhat, vhat = 0.9 * m / (1 - 0.9 ** 7), 0.99 * v / (1 - 0.99 ** 7)
    np.testing.assert_allclose(w1, w - 0.1 * (mhat / (np.sqrt(vhat) + 1e-3) + 0.5 * w), rtol=1e-14)


def test_two_steps_by_hand():
    # scalar, beta1 = 1/2, beta2 = 3/4, eps = 0, lr = 1, no decay, w0 = 0, g1 = 2, g2 = -2
    #  t=1: m = 1, v = 1; mhat = 1 / (1/2) = 2, vhat = 1 / (1/4) = 4 -> w = 0 - 2 / 2 = -1
    #  t=2: m = 1/2 - 1 = -1/2, v = 3/4 + 1 = 7/4; mhat = (-1/2) / (3/4) = -2/3, vhat = (7/4) / (7/16) = 4
    #       -> w = -1 + (2/3) / 2 = -2/3
    w, m, v = ao.adamw_step([0.0], [2.0], [0.0], [0.0], 1, lr=1.0, beta1=0.5, beta2=0.75, eps=0.0)
    assert (w[0], m[0], v[0]) == (-1.0, 1.0, 1.0)
    w, m, v = ao.adamw_step(w, [-2.0], m, v, 2, lr=1.0, beta1=0.5, beta2=0.75, eps=0.0)
    assert m[0] == -0.5 and v[0] == 1.75
    assert abs(w[0] - (-2.0 / 3.0)) < 1e-15


@pytest.mark.parametrize("wd", [0.0, 0.05])
def test_against_torch_cpu(wd):
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(3)
    w0 = rng.normal(size=(7, 5))
    p = torch.nn.Parameter(torch.tensor(w0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=wd)
    w, m, v = w0.copy(), np.zeros_like(w0), np.zeros_like(w0)
    for t in range(1, 6):
        g = rng.normal(size=(7, 5))
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = ao.adamw_step(w, g, m, v, t, lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=wd)
        np.testing.assert_allclose(p.detach().numpy(), w, rtol=1e-12, atol=1e-14)
