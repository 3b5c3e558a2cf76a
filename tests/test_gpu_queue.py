"""GPU parity of the message-queue form (Algorithm 1's server state held literally: one model,
the messages of the last tau_max+1 iterations queued) against the oracle's step-wise queue form,
and against the ring form of the library itself.  Bar as everywhere: bit-exact."""
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


def problem(d, n, seed, noise_kind=1):
    w = workloads.replace(workloads.get("C1", d=d, n=n), seed=seed, noise_kind=noise_kind)
    return (w,) + tuple(workloads.make_problem(w))


def queue_pair(ddef, oracle_mod, w, lam, xstar, x0, tau, tau_max):
    g = ddef.Context(w.d, w.n, tau_max, queue_form=True)
    g.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    g.set_tau(tau)
    o = oracle_mod.QueueOracle(w.d, w.n, tau)
    o.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    return g, o


def assert_same(g, o, n, what):
    for i in range(n):
        gi, gv = g.get_message(i)
        oi, ov = o.get_message(i)
        assert np.array_equal(gi, oi), (what, "indices", i)
        assert np.array_equal(bits(gv), bits(ov)), (what, "values", i)
        assert np.array_equal(bits(g.get_error(i)), bits(o.get_error(i))), (what, "error buffer", i)
    assert np.array_equal(bits(g.get_update()), bits(o.get_update())), (what, "update")
    assert np.array_equal(bits(g.get_model()), bits(o.get_model())), (what, "model")


@pytest.mark.parametrize("tau,delta,d,n", [(0, 0.01, 70001, 3), (1, 0.02, 70001, 3), (3, 0.005, 263171, 2),
                                           (4, 0.3, 9001, 4)])
def test_queue_form_matches_stepwise_oracle(ddef, oracle_mod, tau, delta, d, n):
    w, lam, xstar, x0 = problem(d, n, seed=100 + tau)
    g, o = queue_pair(ddef, oracle_mod, w, lam, xstar, x0, tau, tau_max=tau + 1)
    for t in range(tau + 7):
        g.step(delta, w.lr)
        o.step(delta, w.lr)
        assert_same(g, o, n, (tau, delta, t))
    assert g.full_select_count() < n * (tau + 7)       # the candidate filter took over
    g.close()
    o.close()


def test_queue_form_equals_ring_form_on_the_gpu(ddef):
    tau, delta = 3, 0.01
    w, lam, xstar, x0 = problem(150001, 4, seed=7, noise_kind=2)
    q = ddef.Context(w.d, w.n, tau, queue_form=True)
    r = ddef.Context(w.d, w.n, tau)
    for c in (q, r):
        c.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        c.set_tau(tau)
    for t in range(14):
        q.step(delta, w.lr)
        r.step(delta, w.lr)
        assert np.array_equal(bits(q.get_model()), bits(r.get_model())), t
        assert np.array_equal(bits(q.get_update()), bits(r.get_update())), t
    q.close()
    r.close()
    # what the queue form sends at t is what the ring form computes at t + tau: with the ring
    # form started tau iterations earlier, messages and error buffers coincide
    q = ddef.Context(w.d, w.n, tau, queue_form=True)
    r = ddef.Context(w.d, w.n, tau)
    for c in (q, r):
        c.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        c.set_tau(tau)
    for t in range(tau):
        r.step(delta, w.lr)
    for t in range(6):
        q.step(delta, w.lr)
        r.step(delta, w.lr)
        for i in range(w.n):
            qi, qv = q.get_message(i)
            ri, rv = r.get_message(i)
            assert np.array_equal(qi, ri) and np.array_equal(bits(qv), bits(rv))
            assert np.array_equal(bits(q.get_error(i)), bits(r.get_error(i)))
    q.close()
    r.close()


def test_queue_survives_growing_messages_and_changing_tau(ddef, oracle_mod):
    """delta rises mid-run (the message rows are reallocated while earlier, shorter messages are
    still queued) and falls again; tau moves within [0, tau_max]."""
    w, lam, xstar, x0 = problem(50021, 3, seed=31)
    g, o = queue_pair(ddef, oracle_mod, w, lam, xstar, x0, tau=2, tau_max=3)
    schedule = [(2, 0.01), (2, 0.01), (2, 0.01), (2, 0.2), (2, 0.2), (3, 0.2), (3, 0.5), (1, 0.5),
                (1, 0.004), (0, 0.004), (3, 1.0), (3, 0.01), (2, 0.01), (2, 0.01)]
    for t, (tau, delta) in enumerate(schedule):
        g.set_tau(tau)
        o.set_tau(tau)
        g.step(delta, w.lr)
        o.step(delta, w.lr)
        assert_same(g, o, w.n, (t, tau, delta))
    g.close()
    o.close()


def test_queue_form_fused_gradient_and_non_iid(ddef, oracle_mod):
    tau, delta = 2, 0.01
    w, lam, xstar, x0 = problem(80003, 3, seed=45)
    g, o = queue_pair(ddef, oracle_mod, w, lam, xstar, x0, tau, tau_max=tau)
    g.set_option(ddef.OPT_FUSE_GRAD, 1)
    g.set_heterogeneity(0.5)
    o.set_heterogeneity(0.5)
    for t in range(8):
        g.step(delta, w.lr)
        o.step(delta, w.lr)
        assert_same(g, o, w.n, t)
    g.close()
    o.close()


def test_queue_form_rejects_other_compressors(ddef):
    c = ddef.Context(1000, 2, 1, queue_form=True)
    assert c.raw("set_compressor", ddef.COMPRESSOR_RANDK) == ddef.EINVAL
    assert c.raw("set_compressor", ddef.COMPRESSOR_TOPK) == ddef.OK
    c.close()
