"""Pins for the non-IID variant (Assumption 3: heterogeneous local objectives; Remark on phi and
Section 5.6: phi' replaces phi in DeCo)."""
import numpy as np
import pytest

from paper_2507_17346_amd import workloads

F32 = np.float32


def bits(a):
    return np.asarray(a, dtype=F32).view(np.uint32)


def make(oracle_mod, d, n, tau, zeta, noise_kind=1, noise_scale=0.1, seed=31):
    w = workloads.replace(workloads.get("C1", d=d, n=n), seed=seed, noise_kind=noise_kind, noise_scale=noise_scale)
    lam, xstar, x0 = workloads.make_problem(w)
    o = oracle_mod.Oracle(d, n, tau)
    o.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    o.set_tau(tau)
    o.set_heterogeneity(zeta)
    return o, w, lam, xstar, x0


def local_optima(oracle_mod, w, xstar, zeta):
    return [xstar + F32(zeta) * oracle_mod.noise_fill(w.seed, oracle_mod.HETEROGENEITY_KEY, i, 0, w.d, 1)
            for i in range(w.n)]


def test_zero_heterogeneity_is_the_iid_method(oracle_mod):
    a, w, *_ = make(oracle_mod, 2000, 3, 1, 0.0)
    b, *_ = make(oracle_mod, 2000, 3, 1, 0.0)
    b.set_heterogeneity(0.0)
    for _ in range(6):
        a.step(0.05, 0.05); b.step(0.05, 0.05)
    assert np.array_equal(bits(a.get_model()), bits(b.get_model()))


def test_gradient_uses_the_workers_own_optimum(oracle_mod):
    zeta = 0.7
    o, w, lam, xstar, x0 = make(oracle_mod, 3000, 4, 0, zeta)
    opt = local_optima(oracle_mod, w, xstar, zeta)
    # the shifts are standard normal and differ between workers
    u = np.stack([(opt[i] - xstar) / F32(zeta) for i in range(w.n)]).astype(np.float64)
    assert abs(u.mean()) < 0.03 and abs(u.var() - 1.0) < 0.05
    assert abs(np.corrcoef(u[0], u[1])[0, 1]) < 0.06
    o.grad()
    for i in range(w.n):
        z = oracle_mod.noise_fill(w.seed, 0, i, 0, w.d, 1)
        want = lam * (x0 - opt[i]) + F32(w.noise_scale) * z
        assert np.array_equal(bits(o.get_grad(i)), bits(want))


def test_noiseless_dsgd_converges_to_the_average_optimum(oracle_mod):
    # delta = 1, tau = 0, no noise: x_t - mean_i x*_i = (1 - lr*lambda)^t (x_0 - mean_i x*_i)
    zeta, lr, steps = 0.5, 0.05, 60
    o, w, lam, xstar, x0 = make(oracle_mod, 800, 4, 0, zeta, noise_kind=0, noise_scale=0.0)
    opt = np.mean([v.astype(np.float64) for v in local_optima(oracle_mod, w, xstar, zeta)], axis=0)
    for _ in range(steps):
        o.step(1.0, lr)
    want = opt + (1.0 - lr * lam.astype(np.float64)) ** steps * (x0.astype(np.float64) - opt)
    assert np.abs(o.get_model() - want).max() <= steps * 2.0 ** -21 * np.abs(want).max()
    # the local gradients at the average optimum do not vanish: that is the heterogeneity
    g_at_opt = [lam * (opt.astype(F32) - v) for v in local_optima(oracle_mod, w, xstar, zeta)]
    assert np.mean([np.square(g).sum() for g in g_at_opt]) > 0.0
    assert np.abs(np.mean(g_at_opt, axis=0)).max() < 1e-6


def test_ef_identity_holds_with_heterogeneity(oracle_mod):
    o, w, lam, xstar, x0 = make(oracle_mod, 2500, 3, 2, 0.3)
    lr, delta = 0.05, 0.02
    for t in range(7):
        e_before = [o.get_error(i) for i in range(w.n)]
        o.grad(); o.ef_compress(delta, lr)
        if t >= 2:
            for i in range(w.n):
                idx, val = o.get_message(i)
                p = e_before[i] + F32(lr) * o.get_grad(i)
                assert np.array_equal(bits(val), bits(p[idx]))
                e_after = o.get_error(i)
                mask = np.ones(w.d, dtype=bool); mask[idx] = False
                assert np.all(bits(e_after[idx]) == 0) and np.array_equal(bits(e_after[mask]), bits(p[mask]))
        o.aggregate(); o.apply_delayed()


def test_phi_prime_and_the_non_iid_deco(oracle_mod):
    for delta in [1.0, 0.5, 0.01]:
        for tau in [0, 3, 9]:
            assert oracle_mod.phi_prime(delta, tau) == pytest.approx(oracle_mod.phi(delta, tau) / delta, rel=1e-14)
    assert oracle_mod.phi_prime(1.0, 4) == 0.0
    assert oracle_mod.phi_prime(0.1, 0) == pytest.approx(0.9 / 0.01, rel=1e-14)
    rng = np.random.default_rng(6)
    differs = 0
    for _ in range(300):
        v_g = 32 * 10 ** rng.uniform(6, 9)
        a = 10 ** rng.uniform(8, 10)
        b = rng.uniform(0.01, 0.3)
        t_comp = 10 ** rng.uniform(-2, 0)
        lo, hi = int(np.ceil(b / t_comp)), int(np.ceil((b + v_g / a) / t_comp))
        best = None
        for tau in range(lo, hi + 1):
            delta = min((tau * t_comp - b) * a / v_g, t_comp * a / v_g, 1.0)
            if delta <= 0:
                continue
            obj = (1 - delta) / (delta ** 2 * (1 - delta / 2) ** tau)
            if best is None or obj < best[0]:
                best = (obj, tau, delta)
        got = oracle_mod.deco_noniid(v_g, a, b, t_comp)
        assert (got is None) == (best is None)
        if got:
            assert got[0] == best[1] and got[1] == pytest.approx(best[2], rel=1e-12)
            differs += got != oracle_mod.deco(v_g, a, b, t_comp)
    assert differs > 0          # the stronger penalty on small delta changes some decisions
