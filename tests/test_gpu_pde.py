"""GPU parity of the reaction-diffusion study (Section 5, Appendix B) against the oracle: loss, the sampled
gradient estimate for the same keys, and the number of kept entries, over grids, step counts on both sides of the
kernels' 1024-step tables, fractions, and several problems per launch.  Both sides compute in fp64; they differ
in the order of sums (stencil neighbours, the reduction over nodes), so values agree to about 1e-12 relative and
the tests ask for 1e-9."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import rad_oracle as R


@pytest.fixture(scope="module")
def ctx():
    from paper_2007_10412_amd import binding as B
    c = B.rad_ctx_create()
    yield c
    B.rad_ctx_destroy(c)


def run(ctx, n, steps, p, thetas, seed, stream, D=0.25, dt=1 / 4096):
    from paper_2007_10412_amd import binding as B
    grid = B.make_pde_grid(n, steps, D, dt)
    problems = len(thetas)
    ws = torch.empty(B.rad_pde_workspace_bytes(ctx, grid, p, problems), dtype=torch.uint8, device="cuda")
    th = torch.tensor(np.asarray(thetas), dtype=torch.float64, device="cuda")
    loss = torch.empty(problems, dtype=torch.float64, device="cuda")
    grad = torch.empty(problems, 7, dtype=torch.float64, device="cuda")
    stored = torch.empty(problems, dtype=torch.int64, device="cuda")
    print("pde n=%d steps=%d p=%g problems=%d" % (n, steps, p, problems), flush=True)
    B.rad_pde_gradient(ctx, grid, th, p, seed, stream, ws, loss, grad, stored)
    return loss.cpu().numpy(), grad.cpu().numpy(), stored.cpu().numpy()


@pytest.mark.parametrize("n,steps,p", [(6, 1, 1.0), (6, 2, 0.5), (8, 40, 1.0), (8, 40, 0.3), (16, 300, 0.05),
                                       (32, 1100, 0.1), (5, 2049, 0.5), (32, 64, 1.0)])
def test_matches_the_oracle(ctx, n, steps, p):
    rng = np.random.default_rng(n * 1000 + steps)
    thetas = rng.uniform(-1, 1, (3, 7))
    dt = 1 / 4096 if n > 8 else 1 / 512          # a longer step on small grids, so that C shapes the solution
    loss, grad, stored = run(ctx, n, steps, p, thetas, seed=77, stream=5, dt=dt)
    for q in range(3):
        l_ref, g_ref, s_ref = R.pde_rad_gradient(thetas[q], n, steps, p, 77, stream_id=5 + q, dt=dt)
        assert stored[q] == s_ref, (q, stored[q], s_ref)
        assert abs(loss[q] - l_ref) <= 1e-9 * abs(l_ref), (q, loss[q], l_ref)
        assert np.abs(grad[q] - g_ref).max() <= 1e-9 * np.abs(g_ref).max(), (q, grad[q], g_ref)


def test_paper_grid_full_length(ctx):
    """Appendix B's problem as it is: 32 x 32 intervals, dt = 1/4096, t from 0 to 10 (40960 steps), 1 % of every
    state kept."""
    theta = np.random.default_rng(4).uniform(-1, 1, (1, 7))
    loss, grad, stored = run(ctx, 32, 40960, 0.01, theta, seed=1, stream=0)
    l_ref, g_ref, s_ref = R.pde_rad_gradient(theta[0], 32, 40960, 0.01, 1, stream_id=0)
    assert stored[0] == s_ref
    assert abs(loss[0] - l_ref) <= 1e-9 * abs(l_ref)
    assert np.abs(grad[0] - g_ref).max() <= 1e-9 * np.abs(g_ref).max()
    assert abs(stored[0] / (40961 * 961) - 0.01) < 1e-3          # the memory kept is the fraction asked for


def test_argument_checks(ctx):
    from paper_2007_10412_amd import binding as B
    for grid, p in ((B.make_pde_grid(33, 10), 0.5), (B.make_pde_grid(8, 0), 0.5), (B.make_pde_grid(8, 10), 0.0),
                    (B.make_pde_grid(32, 10, D=1.0, dt=1 / 1024), 0.5)):       # D dt n^2 = 1 > 1/4
        with pytest.raises(B.RadError):
            B.rad_pde_workspace_bytes(ctx, grid, p, 1)
    grid = B.make_pde_grid(8, 10)
    th = torch.zeros(1, 7, dtype=torch.float64, device="cuda")
    out = torch.zeros(8, dtype=torch.float64, device="cuda")
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    with pytest.raises(B.RadError) as e:
        B.rad_pde_gradient(ctx, grid, th, 0.5, 1, 0, small, out, out)
    assert e.value.status == B.RAD_ERR_CAPACITY
