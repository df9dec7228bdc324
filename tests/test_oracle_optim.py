"""Pins of the oracle's parameter updates (Section 4.3 / Appendix A: Adam with l2 regularisation for the
feedforward networks, SGD without momentum for the RNN): torch.optim on the CPU as an independent
implementation, and the closed form of Adam under a constant gradient."""
import numpy as np
import torch

from oracle import rad_oracle as R


def test_sgd_is_torch_sgd_with_weight_decay():
    rng = np.random.default_rng(1)
    w = rng.standard_normal(257)
    tw = torch.tensor(w.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([tw], lr=3e-2, weight_decay=1e-3)
    for step in range(4):
        g = rng.standard_normal(257)
        w = R.sgd_step(w, g, 3e-2, 1e-3)
        tw.grad = torch.tensor(g.copy())
        opt.step()
    np.testing.assert_allclose(w, tw.detach().numpy(), rtol=0, atol=1e-14)


def test_adam_is_torch_adam_with_weight_decay():
    rng = np.random.default_rng(2)
    w = rng.standard_normal(300)
    m = np.zeros(300); v = np.zeros(300)
    tw = torch.tensor(w.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([tw], lr=1e-2, betas=(0.8, 0.95), eps=1e-6, weight_decay=1e-2)
    for t in range(1, 8):
        g = rng.standard_normal(300) * 10.0 ** rng.integers(-3, 2)
        w, m, v = R.adam_step(w, g, m, v, t, 1e-2, 0.8, 0.95, 1e-6, 1e-2)
        tw.grad = torch.tensor(g.copy())
        opt.step()
    np.testing.assert_allclose(w, tw.detach().numpy(), rtol=0, atol=1e-12)


def test_adam_constant_gradient_closed_form():
    # with zero initial moments and a constant gradient both bias-corrected moments are exact at every step
    # (m^ = g, v^ = g^2), so each step moves w by lr g / (|g| + eps)
    g = np.array([2.0, -0.5, 1e-3, 0.0])
    w = np.array([1.0, 1.0, 1.0, 1.0])
    m = np.zeros(4); v = np.zeros(4)
    lr, eps = 0.1, 1e-8
    for t in range(1, 6):
        w, m, v = R.adam_step(w, g, m, v, t, lr, 0.9, 0.999, eps)
        np.testing.assert_allclose(w, 1.0 - t * lr * g / (np.abs(g) + eps), rtol=0, atol=1e-12)


def test_first_adam_step_has_the_size_of_the_learning_rate():
    rng = np.random.default_rng(3)
    g = rng.standard_normal(100) * 1e3
    w, m, v = R.adam_step(np.zeros(100), g, np.zeros(100), np.zeros(100), 1, 1e-3)
    np.testing.assert_allclose(w, -1e-3 * np.sign(g), rtol=1e-6)      # eps against |g| of order 1e3
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-12)
    np.testing.assert_allclose(v, 1e-3 * g * g, rtol=1e-9)
