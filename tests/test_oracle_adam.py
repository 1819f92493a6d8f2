"""Pins of the oracle's weight update (Adam; section V-B-3 Apply, section VI-A optimizer)."""
import numpy as np
import torch

from oracle import stage_oracle as O


def test_adam_matches_an_independent_library_implementation_over_several_steps():
    rng = np.random.default_rng(7)
    n = 257
    theta = rng.normal(0, 0.02, n)
    m, v = np.zeros(n), np.zeros(n)
    p = torch.tensor(theta.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=1e-4, betas=(0.9, 0.999), eps=1e-8)
    for step in range(1, 6):
        G = rng.normal(0, 3.0, n) * (step % 2 + 0.1)
        scale = 1.0 / 32
        theta, m, v = O.adam_apply(theta, m, v, G, step, 1e-4, 0.9, 0.999, 1e-8, scale)
        p.grad = torch.tensor(G * scale)
        opt.step()
        assert np.allclose(theta, p.detach().numpy(), rtol=1e-12, atol=1e-15)


def test_adam_first_step_closed_form_and_zero_gradient():
    g = np.array([3.0, -0.5, 1e-9, 0.0])
    theta = np.array([1.0, 2.0, 3.0, 4.0])
    lr, eps = 0.01, 1e-8
    t1, m1, v1 = O.adam_apply(theta, np.zeros(4), np.zeros(4), g, 1, lr, 0.9, 0.999, eps)
    # bias correction makes m-hat = g and v-hat = g^2 on the first step
    assert np.allclose(t1, theta - lr * g / (np.abs(g) + eps), rtol=1e-12)
    assert np.allclose(m1, 0.1 * g) and np.allclose(v1, 0.001 * g * g)
    assert t1[3] == theta[3]                     # no gradient, no motion
    assert np.all(np.abs(t1 - theta) <= lr)      # a step never exceeds lr on the first update
    # the inputs are not modified
    assert theta[0] == 1.0


def test_adam_grad_scale_is_an_average():
    rng = np.random.default_rng(3)
    G = rng.normal(size=16)
    a = O.adam_apply(np.zeros(16), np.zeros(16), np.zeros(16), G, 1, 1e-3, grad_scale=0.25)
    b = O.adam_apply(np.zeros(16), np.zeros(16), np.zeros(16), 0.25 * G, 1, 1e-3)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
