"""ddef_step with DDEF_OPT_GRAPH: steady iterations are recorded once as a HIP graph and replayed.
Every replay is checked against the oracle (and so against the eager launches), with eager work
of the library itself (getters, which wait for the stream and copy) between the replays."""
import numpy as np
import pytest

from paper_2507_17346_amd import workloads

pytestmark = pytest.mark.gpu

F32 = np.float32


def bits(a):
    return np.asarray(a, dtype=F32).view(np.uint32)


@pytest.fixture(scope="module")
def ddef():
    from paper_2507_17346_amd import binding
    binding.load()
    return binding


def pair(ddef, oracle_mod, w, tau, graph=True, fuse=False):
    lam, xstar, x0 = workloads.make_problem(w)
    g = ddef.Context(w.d, w.n, tau)
    o = oracle_mod.Oracle(w.d, w.n, tau, threads=4)
    for h in (g, o):
        h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        h.set_tau(tau)
    g.set_option(ddef.OPT_GRAPH, 1 if graph else 0)
    g.set_option(ddef.OPT_FUSE_GRAD, 1 if fuse else 0)
    return g, o


def check(g, o, n, what):
    for i in range(n):
        gi, gv = g.get_message(i)
        oi, ov = o.get_message(i)
        assert np.array_equal(gi, oi), (what, "indices", i)
        assert np.array_equal(bits(gv), bits(ov)), (what, "values", i)
        assert np.array_equal(bits(g.get_error(i)), bits(o.get_error(i))), (what, "error buffer", i)
    assert np.array_equal(bits(g.get_update()), bits(o.get_update())), (what, "update")
    assert np.array_equal(bits(g.get_model()), bits(o.get_model())), (what, "model")


@pytest.mark.parametrize("tau,fuse", [(0, False), (3, False), (2, True)])
def test_replayed_iterations_match_the_oracle(ddef, oracle_mod, tau, fuse):
    w = workloads.get("C3", d=300_007, n=4)
    g, o = pair(ddef, oracle_mod, w, tau, fuse=fuse)
    steps = tau + 14
    for t in range(steps):
        g.step(0.002, w.lr)
        o.step(0.002, w.lr)
        check(g, o, w.n, (tau, fuse, t))
    # empty iterations, the whole-row start and the first filtered iteration run eagerly, one
    # iteration records; the rest must have been replays
    assert g.graph_replays() >= steps - tau - 5, g.graph_replays()
    assert g.t == steps
    g.close()
    o.close()


def test_recording_follows_changes_of_k_tau_and_lr(ddef, oracle_mod):
    w = workloads.get("C1", d=90_001, n=3)
    g, o = pair(ddef, oracle_mod, w, 4)
    plan = [(2, 0.01, 0.05)] * 7 + [(2, 0.02, 0.05)] * 5 + [(4, 0.02, 0.05)] * 5 + [(4, 0.02, 0.025)] * 5
    tau_now = None
    for t, (tau, delta, lr) in enumerate(plan):
        if tau != tau_now:
            g.set_tau(tau); o.set_tau(tau)
            tau_now = tau
        g.step(delta, lr)
        o.step(delta, lr)
        check(g, o, w.n, (t, tau, delta, lr))
    assert g.graph_replays() >= 8, g.graph_replays()
    g.close()
    o.close()


def test_mixing_single_calls_and_replays(ddef, oracle_mod):
    """The four calls and ddef_step may alternate; a replay after eager iterations picks up the
    right iteration number (noise key, ring slots)."""
    w = workloads.get("C1", d=50_003, n=2)
    g, o = pair(ddef, oracle_mod, w, 1)
    for t in range(16):
        if t in (7, 8, 12):
            g.grad(); g.ef_compress(0.01, w.lr); g.aggregate(); g.apply_delayed(w.lr)
        else:
            g.step(0.01, w.lr)
        o.step(0.01, w.lr)
        check(g, o, w.n, t)
    assert g.graph_replays() >= 6
    g.close()
    o.close()


def test_without_the_option_nothing_is_recorded(ddef, oracle_mod):
    w = workloads.get("C1", d=20_000, n=2)
    g, o = pair(ddef, oracle_mod, w, 0, graph=False)
    for t in range(6):
        g.step(0.01, w.lr)
        o.step(0.01, w.lr)
    check(g, o, w.n, "eager")
    assert g.graph_replays() == 0
    g.close()
    o.close()
