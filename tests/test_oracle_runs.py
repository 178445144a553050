"""Pins for the oracle's run-level behaviour: the PASGD update rule, the
averaging operator, the quadratic closed forms and the AdaComm driver.  Each
test compares the oracle with an independent statement of the same fact."""
import math

import numpy as np
import pytest

import synth

SEED = 1810_08313


def _small_problem(orc, m=4, dims=(10, 8, 4), B=6, N=200, lr=0.1, beta=0.0, wd=0.0, bf16=False, seed=SEED):
    dims = list(dims)
    data, labels = synth.gaussian_mixture(seed, N, dims[0], dims[-1], mean_sd=1.5)
    x1 = synth.init_params(seed, dims)
    md = orc.make_model(orc.KIND_MLP, dims, B=B, N=N, E=min(N, 64), lr=lr, beta=beta, wd=wd, bf16=bf16)
    run = orc.Run(m, md, seed, x1, data, labels)
    return run, md, data, labels, x1


def _batch(orc, seed, i, k, B, N):
    return [orc.index(seed, i, k, b, N) for b in range(B)]


# ------------------------------------------------------------ PASGD update rule

@pytest.mark.parametrize("beta", [0.0, 0.9])
def test_tau1_is_synchronous_sgd_on_the_mean_gradient(orc, beta):
    """Special case tau = 1 (Sec. 2): x <- x - lr * (1/m) sum_i g(x; xi^(i)).
    With per-worker buffers that all start at zero the same holds for momentum
    by linearity (the mean buffer is the buffer of the mean gradient)."""
    m, B, N, lr = 4, 6, 200, 0.1
    run, md, data, labels, x1 = _small_problem(orc, m=m, B=B, N=N, lr=lr, beta=beta)
    x = x1.astype(np.float64)
    v = np.zeros_like(x)
    for k in range(6):
        gs = []
        for i in range(m):
            _, g = orc.mlp_loss_grad(md, x.astype(np.float32), data, labels, _batch(orc, SEED, i, k, B, N))
            gs.append(g.astype(np.float64))
        v = beta * v + np.mean(gs, axis=0)
        x = x - lr * v
        run.local_steps(1)
        run.average()
        assert np.abs(run.X[0] - x).max() < 2e-6 * np.abs(x).max(), k
    assert run.k == 6


@pytest.mark.parametrize("tau", [1, 3, 7])
def test_single_worker_is_serial_sgd_bit_for_bit(orc, tau):
    """m = 1: the mean over one model is the model, so PASGD is mini-batch SGD."""
    B, N, lr, beta = 6, 200, 0.1, 0.9
    run, md, data, labels, x1 = _small_problem(orc, m=1, B=B, N=N, lr=lr, beta=beta, wd=1e-3)
    x, v = x1.copy(), np.zeros_like(x1)
    k = 0
    for _ in range(3):
        for _ in range(tau):
            _, g = orc.mlp_loss_grad(md, x, data, labels, _batch(orc, SEED, 0, k, B, N))
            orc.sgd_update(x, v, g, lr, beta, 1e-3)
            k += 1
        run.local_steps(tau)
        run.average()
        assert np.array_equal(run.X[0].view(np.uint32), x.view(np.uint32))
        assert np.array_equal(run.V[0].view(np.uint32), v.view(np.uint32))
    assert run.k == k


def test_averaging_rows_identical_mean_preserved_idempotent(orc):
    run, *_ = _small_problem(orc, m=5, beta=0.9)
    run.local_steps(4)
    X0 = run.X.copy()
    V0 = run.V.copy()
    assert np.abs(X0 - X0[0]).max() > 0          # the workers have drifted apart
    run.average()
    X1 = run.X.copy()
    for i in range(1, 5):
        assert np.array_equal(X1[i].view(np.uint32), X1[0].view(np.uint32))
    exact = X0.astype(np.float64).mean(axis=0)
    assert np.abs(X1[0] - exact).max() <= np.abs(np.spacing(exact.astype(np.float32))).max()
    assert np.array_equal(run.V, V0)              # per-worker buffers are not communicated
    run.average()
    assert np.array_equal(run.X.view(np.uint32), X1.view(np.uint32))


def test_spread_identity_inside_a_period(orc):
    """Plain SGD between two averaging steps (Appendix, proof of the variable-tau
    theorem): X_k (I - J) = -lr * sum_r G_r (I - J), i.e. each worker's offset
    from the mean equals -lr times its centred accumulated gradient."""
    m, B, N, lr = 4, 6, 200, 0.05
    run, md, data, labels, x1 = _small_problem(orc, m=m, B=B, N=N, lr=lr)
    acc = np.zeros((m, x1.size))
    for k in range(5):
        Xk = run.X.copy()
        for i in range(m):
            _, g = orc.mlp_loss_grad(md, Xk[i], data, labels, _batch(orc, SEED, i, k, B, N))
            acc[i] += g
        run.local_steps(1)
        lhs = run.X.astype(np.float64) - run.X.astype(np.float64).mean(axis=0)
        rhs = -lr * (acc - acc.mean(axis=0))
        assert np.abs(lhs - rhs).max() < 1e-6 * max(1.0, np.abs(run.X).max()), k


def test_update_from_explicit_gradients(orc):
    m, P = 3, 50
    X, G = synth.flat_stress(3, m, P)
    md = orc.make_model(orc.KIND_QUAD, [P], lr=0.1, beta=0.9, wd=0.01)
    run = orc.Run(m, md, 1, X[0], qa=np.ones((m, P), np.float32), qc=np.zeros((m, P), np.float32))
    run.X[:] = X
    x, v = X.astype(np.float64), np.zeros((m, P))
    for _ in range(3):
        run.update_from_grad(G)
        v = 0.9 * v + (G + 0.01 * x)
        x = x - 0.1 * v
    assert np.abs(run.X - x).max() < 1e-6
    assert np.abs(run.V - v).max() < 1e-6
    assert run.k == 0


# -------------------------------------------------------- quadratic closed forms

@pytest.mark.parametrize("common_a", [True, False])
@pytest.mark.parametrize("tau", [1, 4, 9])
def test_quadratic_plain_sgd_closed_form(orc, common_a, tau):
    """Worker i: g_i(x) = a_i (x - c_i).  One local step is x <- rho_i x +
    (1 - rho_i) c_i with rho_i = 1 - lr a_i; tau steps then averaging is the
    affine map x <- alpha x + bt with alpha = mean_i rho_i^tau and
    bt = mean_i (1 - rho_i^tau) c_i; R rounds give
    alpha^R x0 + bt (1 - alpha^R) / (1 - alpha)."""
    m, P, lr, R = 4, 33, 0.2, 5
    a, c, x0 = synth.quad_problem(2, m, P, common_a=common_a)
    md = orc.make_model(orc.KIND_QUAD, [P], lr=lr)
    run = orc.Run(m, md, 0, x0, qa=a, qc=c)
    for _ in range(R):
        run.local_steps(tau)
        run.average()
    rho = 1.0 - lr * a.astype(np.float64)
    alpha = (rho ** tau).mean(axis=0)
    bt = ((1.0 - rho ** tau) * c).mean(axis=0)
    want = alpha ** R * x0 + bt * (1.0 - alpha ** R) / (1.0 - alpha)
    assert np.abs(run.X[0] - want).max() < 3e-6
    assert run.k == tau * R
    if common_a:
        # equal curvature: the synchronised model is gradient descent on the mean
        # objective, whatever tau is
        cbar = c.astype(np.float64).mean(axis=0)
        assert np.abs(run.X[0] - (cbar + rho[0] ** (tau * R) * (x0 - cbar))).max() < 3e-6


def test_quadratic_momentum_closed_form(orc):
    """With the buffer form v <- beta v + g, x <- x - lr v, the pair (x - c, v) of
    one coordinate evolves by the matrix [[1 - lr a, -lr beta], [a, beta]]."""
    m, P, lr, beta, tau = 3, 17, 0.15, 0.9, 6
    a, c, x0 = synth.quad_problem(4, m, P)
    md = orc.make_model(orc.KIND_QUAD, [P], lr=lr, beta=beta)
    run = orc.Run(m, md, 0, x0, qa=a, qc=c)
    run.local_steps(tau)
    for i in range(m):
        for p in range(P):
            M = np.array([[1 - lr * a[i, p], -lr * beta], [a[i, p], beta]], dtype=np.float64)
            s = np.linalg.matrix_power(M, tau) @ np.array([x0[p] - c[i, p], 0.0])
            assert abs(run.X[i, p] - (c[i, p] + s[0])) < 3e-6
            assert abs(run.V[i, p] - s[1]) < 3e-6
    # averaging leaves the buffers alone and the next period continues from them
    V = run.V.copy()
    run.average()
    xbar = run.X[0].astype(np.float64)
    run.local_steps(2)
    for p in range(P):
        M = np.array([[1 - lr * a[1, p], -lr * beta], [a[1, p], beta]], dtype=np.float64)
        s = np.linalg.matrix_power(M, 2) @ np.array([xbar[p] - c[1, p], V[1, p]])
        assert abs(run.X[1, p] - (c[1, p] + s[0])) < 3e-6


def test_quadratic_loss_closed_form(orc):
    m, P = 4, 21
    a, c, x0 = synth.quad_problem(6, m, P)
    md = orc.make_model(orc.KIND_QUAD, [P], lr=0.1)
    run = orc.Run(m, md, 0, x0, qa=a, qc=c)
    c64 = c.astype(np.float64)
    want = float(np.mean([0.5 * np.sum(a[i].astype(np.float64) * (x0.astype(np.float64) - c64[i]) ** 2)
                          for i in range(m)]))
    assert abs(run.loss() - want) < 1e-12 * want
    run.local_steps(3)
    xbar = run.X.astype(np.float64).mean(axis=0).astype(np.float32).astype(np.float64)
    want = float(np.mean([0.5 * np.sum(a[i].astype(np.float64) * (xbar - c64[i]) ** 2) for i in range(m)]))
    X = run.X.copy()
    assert abs(run.loss() - want) < 1e-12 * want
    assert np.array_equal(run.X, X)                # evaluating the loss changes nothing


def test_mlp_loss_is_mean_cross_entropy_of_the_averaged_model(orc):
    from test_oracle_pieces import _np_loss
    run, md, data, labels, x1 = _small_problem(orc, m=3)
    run.local_steps(2)
    xbar = run.X.astype(np.float64).mean(axis=0).astype(np.float32)
    E = md.E
    want = _np_loss(xbar, list(md.dims[:md.n_layers + 1]), data[:E], labels[:E])
    assert abs(run.loss() - want) < 2e-6 * want


# ------------------------------------------------------------------- the driver

@pytest.mark.parametrize("K,tau", [(12, 4), (13, 4), (5, 8), (9, 1)])
def test_fixed_tau_driver_counts(orc, K, tau):
    run, *_ = _small_problem(orc, m=2)
    sched, rounds = run.run(K, tau)
    assert sched == [(0, tau)]
    assert rounds == math.ceil(K / tau)           # the last period is truncated
    assert run.k == K
    assert np.array_equal(run.X[0], run.X[1])      # and still ends with an average


def test_driver_equals_manual_loop(orc):
    a = _small_problem(orc, m=3, beta=0.9)[0]
    b = _small_problem(orc, m=3, beta=0.9)[0]
    a.run(10, 4)
    for t in (4, 4, 2):
        b.local_steps(t)
        b.average()
    assert np.array_equal(a.X.view(np.uint32), b.X.view(np.uint32))
    assert np.array_equal(a.V.view(np.uint32), b.V.view(np.uint32))


def test_adaptive_schedule_on_quadratic_follows_the_closed_form(orc):
    """Common curvature, plain SGD: at every averaging step x = cbar + rho^k (x0 -
    cbar) for any tau, so F at each decision point is known in closed form and
    the whole tau schedule can be predicted without running the oracle:
    tau_l = ceil(sqrt(F_l / F_0) tau_0), decisions at the first averaging
    boundary at or after each multiple of the interval (Sec. 4.2, basic rule;
    fixed learning rate, so the sequence is non-increasing, Sec. 4.1)."""
    m, P, lr, tau0, I, K = 4, 16, 0.02, 12, 20, 150
    a, c, x0 = synth.quad_problem(8, m, P, common_a=True)
    c = (c * 0.05).astype(np.float32)               # small floor so that the loss really decays
    md = orc.make_model(orc.KIND_QUAD, [P], lr=lr)
    run = orc.Run(m, md, 0, x0, qa=a, qc=c)
    sched, rounds = run.run(K, tau0, adaptive=True, interval=I)

    a64, c64 = a.astype(np.float64), c.astype(np.float64)
    cbar, rho = c64.mean(axis=0), 1.0 - lr * a64[0]

    def F(k):
        x = cbar + rho ** k * (x0 - cbar)
        return float(np.mean([0.5 * np.sum(a64[i] * (x - c64[i]) ** 2) for i in range(m)]))

    k, tau, next_eval, want, r = 0, tau0, I, [(0, tau0)], 0
    while k < K:
        k += min(tau, K - k)
        r += 1
        if k >= next_eval and k < K:
            p = math.sqrt(F(k) / F(0)) * tau0
            assert abs(p - round(p)) > 1e-3, "decision too close to an integer for this pin"
            tau = max(1, math.ceil(p))
            want.append((k, tau))
            while next_eval <= k:
                next_eval += I
    assert sched == want
    assert rounds == r
    taus = [t for _, t in sched]
    assert taus == sorted(taus, reverse=True) and taus[-1] < tau0
