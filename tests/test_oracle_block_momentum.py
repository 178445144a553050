"""Pins for the oracle's block momentum (Sec. 5.3.1)."""
import numpy as np
import pytest

import synth
from test_oracle_runs import SEED, _batch, _small_problem


def test_zero_global_momentum_is_plain_periodic_averaging(orc):
    """beta_glob = 0 and plain local SGD: u = G, x_sync - lr G = x_bar."""
    a = _small_problem(orc, m=3)[0]
    b = _small_problem(orc, m=3)[0]
    b.block_begin(0.0)
    for _ in range(4):
        a.local_steps(3)
        a.average()
        b.local_steps(3)
        b.average()
        scale = np.abs(a.X).max()
        assert np.abs(a.X - b.X).max() <= 4 * np.spacing(np.float32(scale))
        assert np.array_equal(b.X[0], b.X[1]) and np.array_equal(b.X[0], b.X[2])


def test_tau1_is_synchronous_sgd_with_global_momentum(orc):
    """tau = 1, no local momentum: u <- beta u + mean gradient, x <- x - lr u, i.e.
    ordinary momentum SGD on the m-fold batch with factor beta_glob."""
    m, B, N, lr, bg = 4, 6, 200, 0.1, 0.3
    run, md, data, labels, x1 = _small_problem(orc, m=m, B=B, N=N, lr=lr)
    run.block_begin(bg)
    x, u = x1.astype(np.float64), np.zeros(x1.size)
    for k in range(6):
        gs = [orc.mlp_loss_grad(md, x.astype(np.float32), data, labels, _batch(orc, SEED, i, k, B, N))[1].astype(np.float64)
              for i in range(m)]
        u = bg * u + np.mean(gs, axis=0)
        x = x - lr * u
        run.local_steps(1)
        run.average()
        assert np.abs(run.X[0] - x).max() < 3e-6 * np.abs(x).max(), k
        assert np.abs(run.block_u - u).max() < 1e-4 * max(1.0, np.abs(u).max()), k


@pytest.mark.parametrize("tau", [1, 5])
def test_quadratic_closed_form(orc, tau):
    """Common curvature, plain local SGD: with e_j = x_sync - cbar the period gives
    x_bar - cbar = rho^tau e_j, so G_j = (1 - rho^tau) e_j / lr, u_j = beta u_{j-1} + G_j,
    e_{j+1} = e_j - lr u_j: a two-term linear recurrence per coordinate."""
    m, P, lr, bg, R = 4, 29, 0.1, 0.3, 7
    a, c, x0 = synth.quad_problem(12, m, P, common_a=True)
    run = orc.Run(m, orc.make_model(orc.KIND_QUAD, [P], lr=lr), 0, x0, qa=a, qc=c)
    run.block_begin(bg)
    a64, cbar = a[0].astype(np.float64), c.astype(np.float64).mean(axis=0)
    rho_t = (1.0 - np.float64(np.float32(lr)) * a64) ** tau
    e, u = x0.astype(np.float64) - cbar, np.zeros(P)
    for _ in range(R):
        run.local_steps(tau)
        run.average()
        u = bg * u + (1.0 - rho_t) * e / np.float64(np.float32(lr))
        e = e - np.float64(np.float32(lr)) * u
        assert np.abs(run.X[0] - (cbar + e)).max() < 5e-6
        assert np.abs(run.block_u - u).max() < 5e-5 * max(1.0, np.abs(u).max())
    assert run.k == tau * R


def test_local_buffers_are_cleared_at_every_averaging_step(orc):
    run, md, data, labels, x1 = _small_problem(orc, m=2, beta=0.9)
    run.block_begin(0.3)
    run.local_steps(3)
    assert np.abs(run.V).max() > 0
    run.average()
    assert np.abs(run.V).max() == 0.0
    # so the first step of the next period is a plain SGD step from the synchronised model
    xs = run.X[0].copy()
    run.local_steps(1)
    for i in range(2):
        _, g = orc.mlp_loss_grad(md, xs, data, labels, _batch(orc, SEED, i, 3, md.B, md.N))
        assert np.array_equal(run.V[i], g)
        assert np.abs(run.X[i] - (xs.astype(np.float64) - 0.1 * g)).max() < 1e-6
    # leaving the mode restores plain averaging
    run.block_end()
    run.local_steps(2)
    X = run.X.astype(np.float64).copy()
    V = run.V.copy()
    run.average()
    assert np.abs(run.X[0] - X.mean(axis=0)).max() < 1e-6
    assert np.array_equal(run.V, V)
