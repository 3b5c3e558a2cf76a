"""Pins for the oracle's objective value f(x_t) = (1/n) sum_i f_i(x_t) (Section 2.1, problem (1),
on the synthetic quadratics): tied to the oracle's own (separately pinned) gradient through finite
differences, to the optimum, and to the closed form of noiseless D-SGD."""
import numpy as np
import pytest

from paper_2507_17346_amd import workloads

F32 = np.float32


def make(oracle_mod, d, n, zeta=0.0, seed=5, noise_kind=0, noise_scale=0.0, tau=0):
    w = workloads.replace(workloads.get("C1", d=d, n=n), seed=seed, noise_kind=noise_kind, noise_scale=noise_scale)
    lam, xstar, x0 = workloads.make_problem(w)
    o = oracle_mod.Oracle(d, n, max(tau, 1))
    o.set_problem(lam, xstar, x0, w.seed, noise_kind, noise_scale)
    o.set_tau(tau)
    o.set_heterogeneity(zeta)
    return o, w, lam, xstar, x0


def test_zero_at_the_shared_optimum_and_positive_elsewhere(oracle_mod):
    o, w, lam, xstar, x0 = make(oracle_mod, 3000, 4)
    assert o.objective() > 0.0
    o.set_model(xstar)
    assert o.objective() == 0.0
    # one coordinate off by 2 with curvature lambda_j: f = lambda_j * 4 / 2
    x = xstar.copy()
    x[17] = xstar[17] + F32(2.0)
    o.set_model(x)
    moved = float(x[17]) - float(xstar[17])
    assert o.objective() == pytest.approx(0.5 * float(lam[17]) * moved * moved, rel=1e-12)


@pytest.mark.parametrize("zeta", [0.0, 0.7])
def test_finite_differences_give_the_average_gradient(oracle_mod, zeta):
    # grad f(x) = (1/n) sum_i grad f_i(x): the noiseless gradients the oracle itself produces
    d, n = 500, 3
    o, w, lam, xstar, x0 = make(oracle_mod, d, n, zeta=zeta)
    o.grad()
    g = np.mean([o.get_grad(i).astype(np.float64) for i in range(n)], axis=0)
    for j in [0, 1, 77, 250, d - 1]:
        xp, xm = x0.copy(), x0.copy()
        xp[j] = x0[j] + F32(0.25)
        xm[j] = x0[j] - F32(0.25)
        o.set_model(xp); fp = o.objective()
        o.set_model(xm); fm = o.objective()
        slope = (fp - fm) / (float(xp[j]) - float(xm[j]))         # exact for a quadratic, at the midpoint
        mid = 0.5 * (float(xp[j]) + float(xm[j]))
        want = g[j] + float(lam[j]) * (mid - float(x0[j]))
        # f is a sum of d terms of which the difference keeps one: cancellation costs about d ulps of f
        assert slope == pytest.approx(want, rel=1e-6, abs=1e-9 * fp)
    o.set_model(x0)


def test_heterogeneous_optima_lift_the_minimum(oracle_mod):
    # with zeta != 0 no x makes every f_i zero: at the average optimum f = (1/2n) sum_j lambda_j sum_i (x*_ij - mean)^2
    d, n, zeta = 800, 4, 0.5
    o, w, lam, xstar, x0 = make(oracle_mod, d, n, zeta=zeta)
    u = np.stack([oracle_mod.noise_fill(w.seed, 2 ** 64 - 2, i, 0, d, 1) for i in range(n)])
    opt = xstar[None, :] + F32(zeta) * u
    mean_opt = opt.astype(np.float64).mean(axis=0).astype(F32)
    o.set_model(mean_opt)
    want = 0.5 * np.sum(lam.astype(np.float64) * np.mean((mean_opt.astype(np.float64)[None, :] - opt.astype(np.float64)) ** 2, axis=0))
    assert o.objective() == pytest.approx(want, rel=1e-12)
    # and moving away from it only increases f
    o.set_model(mean_opt + F32(0.01))
    assert o.objective() > want


def test_noiseless_dsgd_follows_the_closed_form(oracle_mod):
    d, n, lr = 2000, 4, 0.05
    o, w, lam, xstar, x0 = make(oracle_mod, d, n)
    lam64, gap0 = lam.astype(np.float64), (x0.astype(np.float64) - xstar.astype(np.float64))
    for t in range(40):
        want = 0.5 * np.sum(lam64 * ((1.0 - float(F32(lr)) * lam64) ** (2 * t)) * gap0 ** 2)
        assert o.objective() == pytest.approx(want, rel=2e-5)
        o.step(1.0, lr)


def test_objective_scales_with_the_curvature(oracle_mod):
    d, n = 1000, 2
    o, w, lam, xstar, x0 = make(oracle_mod, d, n)
    f1 = o.objective()
    o.set_problem(lam * F32(2.0), xstar, x0, w.seed, 0, 0.0)
    assert o.objective() == pytest.approx(2.0 * f1, rel=1e-12)
