"""Pins for the oracle's AdaComm refinements (Sec. 4.3): faster decay when the
loss saturates, the practical learning-rate coupling, and postponing scheduled
learning-rate changes until tau has reached 1."""
import math

import numpy as np
import pytest

import synth


def test_reduces_to_the_basic_rule(orc):
    g = np.random.default_rng(0)
    for _ in range(2000):
        F0, Fl, tau0 = float(g.uniform(0.1, 3)), float(g.uniform(0, 3)), int(g.integers(1, 60))
        basic = orc.next_tau(F0, Fl, tau0)
        # equal learning rates, previous period far above the candidate: the candidate is taken
        assert orc.next_tau_ex(F0, Fl, tau0, 10**6, 0.5, 0, 0.3, 0.3) == basic
        # first decision after a learning-rate change with equal rates: likewise
        assert orc.next_tau_ex(F0, Fl, tau0, 1, 0.5, 0, 0.3, 0.3, lr_changed=True) == basic


def test_saturated_loss_halves_the_period(orc):
    # a loss that does not move gives the same candidate every time, which is never
    # strictly below the current period: gamma = 1/2 halves it down to 1 (Sec. 4.3.1)
    tau, seen = 20, []
    for _ in range(7):
        tau = orc.next_tau_ex(2.0, 2.0, 20, tau, 0.5, 0)
        seen.append(tau)
    assert seen == [10, 5, 3, 2, 1, 1, 1]
    # a smaller gamma decays faster
    assert orc.next_tau_ex(2.0, 2.0, 20, 20, 0.25, 0) == 5


def test_candidate_taken_only_if_strictly_smaller(orc):
    # candidate ceil(sqrt(0.25) * 20) = 10
    assert orc.next_tau_ex(1.0, 0.25, 20, 11) == 10          # 10 < 11
    assert orc.next_tau_ex(1.0, 0.25, 20, 10) == 5           # not strictly smaller: gamma * 10
    assert orc.next_tau_ex(1.0, 0.25, 20, 9) == 5            # ceil(4.5)
    # slack s: the candidate must satisfy c + s < tau_prev
    assert orc.next_tau_ex(1.0, 0.25, 20, 12, 0.5, 1) == 10  # 11 < 12
    assert orc.next_tau_ex(1.0, 0.25, 20, 11, 0.5, 1) == 6   # 11 < 11 fails: ceil(5.5)
    for bad in [dict(gamma=0.0), dict(gamma=1.0), dict(gamma=1.5), dict(slack=-1), dict(lr0=0.0), dict(lrl=-1.0)]:
        kw = dict(gamma=0.5, slack=0, lr0=1.0, lrl=1.0)
        kw.update(bad)
        assert orc.next_tau_ex(1.0, 0.5, 20, 20, **kw) < 0
    assert orc.next_tau_ex(1.0, 0.5, 20, 0) < 0


def test_learning_rate_coupling_closed_forms_and_exact_arithmetic(orc):
    # tau proportional to sqrt(lr0 / lrl) (Sec. 4.3.2): a 4x smaller rate doubles the period
    assert orc.next_tau_ex(1.0, 1.0, 10, 1, 0.5, 0, 0.4, 0.1, lr_changed=True) == 20
    assert orc.next_tau_ex(1.0, 0.25, 10, 1, 0.5, 0, 0.4, 0.1, lr_changed=True) == 10
    # candidate = least n with n^2 F0 q >= tau0^2 Fl p for lr0/lrl = p/q (exactly representable ratios)
    checked = 0
    for F0 in range(1, 12):
        for Fl in range(0, 16):
            for tau0 in (1, 7, 20):
                for p, q in ((1, 1), (2, 1), (4, 1), (8, 1), (1, 2), (16, 1)):
                    exact = math.sqrt(tau0 * tau0 * Fl * p / (F0 * q))
                    if abs(exact - round(exact)) < 1e-9:
                        continue
                    n = max(1, math.ceil(exact))
                    assert (n * n * F0 * q >= tau0 * tau0 * Fl * p) and (n == 1 or (n - 1) ** 2 * F0 * q < tau0 * tau0 * Fl * p)
                    got = orc.next_tau_ex(float(F0), float(Fl), tau0, 1, 0.5, 0, float(p), float(q), lr_changed=True)
                    assert got == n, (F0, Fl, tau0, p, q)
                    checked += 1
    assert checked > 2000


def _quad(orc, lr, seed=8, m=4, P=16):
    a, c, x0 = synth.quad_problem(seed, m, P, common_a=True)
    c = (c * 0.05).astype(np.float32)
    md = orc.make_model(orc.KIND_QUAD, [P], lr=lr)
    return orc.Run(m, md, 0, x0, qa=a, qc=c), a.astype(np.float64), c.astype(np.float64), x0.astype(np.float64)


@pytest.mark.parametrize("postpone", [True, False])
def test_refined_driver_on_quadratic_follows_the_closed_form(orc, postpone):
    """Common curvature, plain SGD: at every averaging step x - cbar is the start
    offset times the product of (1 - lr_j a) over all iterations so far, whatever
    tau was, so the loss at every decision and hence the whole (k, tau, lr)
    sequence can be predicted without the oracle."""
    lr0, tau0, I, K = 0.02, 12, 20, 260
    sched_lr = [(70, 0.005)]
    run, a, c, x0 = _quad(orc, lr0)
    got, rounds = run.run_ex(K, tau0, I, refine=True, gamma=0.5, slack=0, lr_schedule=sched_lr, postpone_lr=postpone)
    m = a.shape[0]
    cbar = c.mean(axis=0)

    def F(off):
        x = cbar + off
        return float(np.mean([0.5 * np.sum(a[i] * (x - c[i]) ** 2) for i in range(m)]))

    off = x0 - cbar
    F0 = F(off)
    k, tau, lr, next_eval, nxt, changed, r = 0, tau0, lr0, I, 0, False, 0
    want = [(0, tau0, pytest.approx(lr0))]
    while k < K:
        t = min(tau, K - k)
        off = off * (1.0 - np.float32(lr).astype(np.float64) * a[0]) ** t
        k += t
        r += 1
        while nxt < len(sched_lr) and k >= sched_lr[nxt][0] and (not postpone or tau == 1):
            lr = sched_lr[nxt][1]
            nxt += 1
            changed = True
        if k >= next_eval and k < K:
            p = math.sqrt((np.float32(lr0).astype(np.float64) / np.float32(lr).astype(np.float64)) * F(off) / F0) * tau0
            assert abs(p - round(p)) > 1e-3, "decision too close to an integer for this pin"
            cand = max(1, math.ceil(p))
            if changed or cand < tau:
                tau = cand
            else:
                tau = max(1, math.ceil(0.5 * tau))
            changed = False
            want.append((k, tau, pytest.approx(lr)))
            while next_eval <= k:
                next_eval += I
    assert got == want
    assert rounds == r and run.k == K
    taus = [t for _, t, _ in got]
    lrs = [l for _, _, l in got]
    assert lrs[-1] == pytest.approx(0.005)
    if postpone:
        # the rate changes only once tau has come down to 1, and the period grows again after it
        first = next(i for i, l in enumerate(lrs) if l == pytest.approx(0.005))
        assert taus[first - 1] == 1 and taus[first] > 1
    else:
        first = next(i for i, l in enumerate(lrs) if l == pytest.approx(0.005))
        assert got[first][0] < 100


def test_refined_driver_without_refinement_equals_basic_driver(orc):
    a, _, _, _ = _quad(orc, 0.02)
    b, _, _, _ = _quad(orc, 0.02)
    sa, ra = a.run(150, 12, adaptive=True, interval=20)
    sb, rb = b.run_ex(150, 12, 20, refine=False)
    assert [(k, t) for k, t, _ in sb] == sa and ra == rb
    assert np.array_equal(a.X, b.X)
