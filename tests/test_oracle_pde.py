"""Pins of the oracle's reaction-diffusion study (Section 5, Appendix B)."""
import numpy as np
import torch

from oracle import rad_oracle as R


def test_stability_number_of_the_paper():
    # Appendix B: dx = 1/32, dt = 1/4096, D = 1/4 satisfy D dt / dx^2 <= 1/4
    assert 0.25 * (1 / 4096) * 32 * 32 == 1 / 16


def test_eigenfunction_decay_closed_form():
    """sin(pi x) sin(pi y) is an eigenvector of the five-point stencil with eigenvalue 4 cos(pi dx) - 4, so with
    C = theta_0 constant every step multiplies phi by rho = 1 + r (4 cos(pi/n) - 4) + dt theta_0."""
    n, steps, dt = 16, 50, 1 / 4096
    for th0 in (0.0, 3.0):
        theta = np.array([th0, 0, 0, 0, 0, 0, 0.0])
        phis, _ = R.pde_forward(theta, n, steps)
        rho = 1 + 0.25 * dt * n * n * (4 * np.cos(np.pi / n) - 4) + dt * th0
        np.testing.assert_allclose(phis[steps], phis[0] * rho**steps, rtol=0, atol=1e-13)
    assert np.all(phis[:, 0, :] == 0) and np.all(phis[:, :, n] == 0)


def test_basis_and_target_at_known_times():
    b = R.pde_basis(8, 0.5)                      # sin(pi t) = 1, cos(pi t) = 0
    x = np.arange(9) / 8
    np.testing.assert_allclose(b[1], 1.0); np.testing.assert_allclose(b[2], 0.0, atol=1e-16)
    np.testing.assert_allclose(b[3], np.sin(2 * np.pi * x), atol=1e-15)
    np.testing.assert_allclose(b[6], 0.0, atol=1e-15)
    phi0 = R.pde_phi0(8)
    assert np.array_equal(R.pde_target(8, 0.0, phi0), phi0) and np.array_equal(R.pde_target(8, 2.0, phi0)[0], phi0[0])
    tg = R.pde_target(8, 0.5, phi0)
    assert abs(tg[2, 4] - (phi0[2, 4] + 0.25 * np.sin(np.pi / 2) * 1.0)) < 1e-15      # x = 1/4, y = 1/2


def _loss_torch(theta, n, steps, dt=1 / 4096, D=0.25):
    r = D * dt * n * n
    x = torch.arange(n + 1, dtype=torch.float64) / n
    phi0 = torch.outer(torch.sin(torch.pi * x), torch.sin(torch.pi * x))
    inner = torch.zeros(n + 1, n + 1, dtype=torch.float64); inner[1:-1, 1:-1] = 1
    phi0 = phi0 * inner
    s2, c2 = torch.sin(2 * torch.pi * x), torch.cos(2 * torch.pi * x)
    phi, loss = phi0, 0.0
    for t in range(steps):
        tt = t * dt
        s, c = np.sin(np.pi * tt), np.cos(np.pi * tt)
        C = theta[0] + theta[1] * s + theta[2] * c + theta[3] * s2 * s + theta[4] * s2 * c + theta[5] * c2 * s + theta[6] * c2 * c
        lap = torch.zeros_like(phi)
        lap[1:-1, 1:-1] = phi[2:, 1:-1] + phi[:-2, 1:-1] + phi[1:-1, 2:] + phi[1:-1, :-2] - 4 * phi[1:-1, 1:-1]
        phi = (phi + r * lap + dt * C[:, None] * phi) * inner
        tg = (phi0 + 0.25 * np.sin(np.pi * (t + 1) * dt) * torch.outer(s2, torch.sin(torch.pi * x))) * inner
        loss = loss + ((phi - tg) ** 2).sum()
    return loss / steps


def test_full_fraction_is_the_exact_gradient():
    rng = np.random.default_rng(1)
    theta = rng.uniform(-1, 1, 7)
    n, steps = 8, 40
    loss, g, stored = R.pde_rad_gradient(theta, n, steps, 1.0, seed=3)
    assert stored == (steps + 1) * (n - 1) ** 2
    tt = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
    lt = _loss_torch(tt, n, steps)
    lt.backward()
    assert abs(loss - lt.item()) < 1e-14
    np.testing.assert_allclose(g, tt.grad.numpy(), rtol=1e-10, atol=1e-16)
    # and against central differences of the oracle's own loss, with a large time step so that C matters
    eps = 1e-6
    for k in range(7):
        e = np.zeros(7); e[k] = eps
        fd = (R.pde_forward(theta + e, n, steps)[1] - R.pde_forward(theta - e, n, steps)[1]) / (2 * eps)
        assert abs(fd - g[k]) < 1e-8 * max(1.0, abs(g[k])) + 1e-9


def test_estimator_is_unbiased():
    rng = np.random.default_rng(2)
    theta = rng.uniform(-1, 1, 7)
    n, steps, p, S = 6, 12, 0.3, 3000
    _, exact, _ = R.pde_rad_gradient(theta, n, steps, 1.0, seed=0)
    est = np.array([R.pde_rad_gradient(theta, n, steps, p, seed=s)[1] for s in range(S)])
    mean, sem = est.mean(axis=0), est.std(axis=0) / np.sqrt(S)
    assert np.all(sem > 0)
    assert np.all(np.abs(mean - exact) < 4.5 * sem), (mean, exact, sem)
    # the stored fraction is p
    stored = R.pde_rad_gradient(theta, n, steps, p, seed=1)[2]
    tot = (steps + 1) * (n - 1) ** 2
    assert abs(stored - p * tot) < 5 * np.sqrt(tot * p * (1 - p))


def test_keep_mask_addressing():
    n, t, p = 5, 7, 0.5
    m = R.pde_keep_mask(n, t, p, seed=9, stream_id=2)
    keys = R.element_keys(9, 2, t, 0, 16)
    assert not m[0].any() and not m[:, n].any()
    for i in range(1, n):
        for j in range(1, n):
            assert m[i, j] == (int(keys[(i - 1) * (n - 1) + (j - 1)]) < 2**31)
