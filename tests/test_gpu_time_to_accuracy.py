"""GPU: the objective value against the oracle's, and the paper's central claim on the synthetic
quadratic: with the timing model of Section 4.1, DeCo's joint choice of staleness and compression
reaches a target objective sooner than D-SGD, compression alone or delay alone (Section 5.3)."""
import numpy as np
import pytest

from paper_2507_17346_amd import time_to_accuracy as tta
from paper_2507_17346_amd import workloads

pytestmark = pytest.mark.gpu

F32 = np.float32


@pytest.fixture(scope="module")
def ddef():
    from paper_2507_17346_amd import binding
    binding.load()
    return binding


@pytest.mark.parametrize("d,n,zeta", [(1, 1, 0.0), (5, 3, 0.0), (4097, 2, 0.3), (300_001, 4, 0.0), (1_000_003, 3, 0.5)])
def test_objective_matches_the_oracle(ddef, oracle_mod, d, n, zeta):
    w = workloads.replace(workloads.get("C1", d=d, n=n), seed=300 + d)
    lam, xstar, x0 = workloads.make_problem(w)
    g = ddef.Context(d, n, 2)
    o = oracle_mod.Oracle(d, n, 2, threads=4)
    for h in (g, o):
        h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        h.set_tau(1)
        h.set_heterogeneity(zeta)
    for t in range(5):
        # double sums in different orders: d terms of similar size
        assert g.objective() == pytest.approx(o.objective(), rel=1e-12 * max(1.0, np.sqrt(d)))
        g.step(0.1, w.lr); o.step(0.1, w.lr)
    g.set_model(xstar)
    if zeta == 0.0:
        assert g.objective() == 0.0
    g.close()


def test_objective_argument_and_state_checks(ddef):
    import ctypes as C
    c = ddef.Context(1000, 2, 1)
    f = C.c_double()
    assert c.raw("objective", C.byref(f)) == ddef.ESTATE          # no problem yet
    one = np.ones(1000, dtype=F32)
    c.set_problem(one, one, one * F32(3.0), 0, 0, 0.0)
    assert c.raw("objective", None) == ddef.EINVAL
    assert c.objective() == pytest.approx(0.5 * 1000 * 4.0)
    c.close()


def test_deco_reaches_the_target_first(ddef):
    w = workloads.get("C1", d=200_000, n=4)
    net = tta.Network(32.0 * w.d, 20e6, 0.1, 0.02)        # V_g / a = 0.32 s, b = 0.1 s, T_comp = 0.02 s
    outcomes = {o.strategy.name: o for o in tta.compare(w, net, target_ratio=0.02, max_iterations=20000,
                                                        check_every=25, tau_max=16)}
    for name, o in outcomes.items():
        assert o.iterations is not None, (name, o.curve[-1])
        print(f"{name:18s} tau={o.strategy.tau:2d} delta={o.strategy.delta:.4f} T_avg={o.t_avg_s:.4f} s "
              f"iterations={o.iterations} seconds={o.seconds:.1f}")
    deco = outcomes["DeCo"]
    for name in ("D-SGD", "compression only", "delay only"):
        assert deco.seconds < outcomes[name].seconds, name
    # compression and delay cost iterations, but far fewer than the time per iteration they save
    assert deco.iterations >= outcomes["D-SGD"].iterations
    assert outcomes["D-SGD"].seconds / deco.seconds > 3.0
    # every curve decreases to its target
    for o in outcomes.values():
        assert o.curve[-1][2] <= 0.02 < o.curve[0][2]


def test_adapting_to_a_changing_network_beats_a_fixed_choice(ddef):
    """Algorithm 2 on a bandwidth that alternates between 200 and 10 Mbit/s every 50 iterations: the
    choice made for the fast period sends 20 times too much in the slow ones."""
    w = workloads.get("C1", d=200_000, n=4)
    v_g = 32.0 * w.d
    nets = [tta.Network(v_g, 200e6, 0.1, 0.02), tta.Network(v_g, 10e6, 0.1, 0.02)]
    fixed = tta.run_adaptive(w, nets, 50, False, 0.02, 20000)
    adaptive = tta.run_adaptive(w, nets, 50, True, 0.02, 20000)
    assert fixed.iterations is not None and adaptive.iterations is not None
    print(f"fixed: {fixed.iterations} iterations, {fixed.seconds:.1f} s; adaptive: {adaptive.iterations} iterations, "
          f"{adaptive.seconds:.1f} s")
    assert adaptive.seconds < fixed.seconds
    # the adaptive run pays about T_comp per iteration throughout
    assert adaptive.seconds / adaptive.iterations == pytest.approx(0.02, rel=0.25)


def test_the_lookup_table_serves_the_adaptive_run(ddef):
    """Section 4.5: (tau, delta) from the nearest of 20 precomputed bandwidths instead of Algorithm 3
    at run time.  Bandwidths between two sample points get a neighbouring choice; the run stays
    close to the one that solves Algorithm 3 every period."""
    w = workloads.get("C1", d=200_000, n=4)
    v_g = 32.0 * w.d
    nets = [tta.Network(v_g, a, 0.1, 0.02) for a in (180e6, 12e6, 60e6, 25e6)]
    lut = ddef.DecoLut(v_g, 10e6, 200e6, 20, 0.1, 0.02)
    direct = tta.run_adaptive(w, nets, 50, True, 0.02, 20000)
    table = tta.run_adaptive(w, nets, 50, True, 0.02, 20000, lut=lut)
    lut.close()
    assert direct.iterations is not None and table.iterations is not None
    print(f"Algorithm 3 every period: {direct.iterations} iterations, {direct.seconds:.2f} s; "
          f"look-up table: {table.iterations} iterations, {table.seconds:.2f} s")
    assert table.seconds == pytest.approx(direct.seconds, rel=0.25)
    assert table.seconds / table.iterations < 0.03
