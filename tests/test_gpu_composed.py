"""GPU parity of the composed compressor (Random-k, Top-k inside the kept coordinates, 4-bit block
codes; Section 5.2 "Baselines") with the oracle, through the C-ABI: index sets, packed codes and
block steps byte for byte, decoded values, error buffers, thresholds, update and model bit for bit."""
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


def pair(ddef, oracle_mod, w, tau, rand_ratio, threads=4):
    lam, xstar, x0 = workloads.make_problem(w)
    g = ddef.Context(w.d, w.n, max(tau, 1))
    o = oracle_mod.Oracle(w.d, w.n, max(tau, 1), threads=threads)
    for h in (g, o):
        h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        h.set_tau(tau)
        h.set_compressor(2)
        h.set_composed(rand_ratio)
    return g, o


def assert_same(g, o, n, what, codes=True):
    for i in range(n):
        gi, gv = g.get_message(i)
        oi, ov = o.get_message(i)
        assert np.array_equal(gi, oi), (what, "indices", i)
        assert np.array_equal(bits(gv), bits(ov)), (what, "decoded values", i)
        if codes and len(oi):
            gc, gs = g.get_message_codes(i)
            oc, os_ = o.get_message_codes(i)
            assert np.array_equal(gc, oc), (what, "codes", i)
            assert np.array_equal(bits(gs), bits(os_)), (what, "steps", i)
            assert g.get_threshold(i) == o.get_threshold(i), (what, "threshold", i)
        assert np.array_equal(bits(g.get_error(i)), bits(o.get_error(i))), (what, "error buffer", i)
    assert np.array_equal(bits(g.get_update()), bits(o.get_update())), what
    assert np.array_equal(bits(g.get_model()), bits(o.get_model())), what


@pytest.mark.parametrize("d,n,tau,rho,delta,steps", [
    (1, 1, 0, 0.2, 0.1, 3),                 # k1 = k = 1
    (3, 2, 0, 0.2, 0.1, 4),
    (33, 3, 1, 0.5, 0.5, 5),                # odd k: the last byte holds one code
    (4097, 2, 2, 0.2, 0.1, 6),
    (100_003, 4, 1, 0.2, 0.1, 6),           # k = 2001: eight blocks, a ragged last one
    (250_000, 8, 1, 0.2, 0.1, 6),           # the paper's ratios and tau = 1
    (65_536, 2, 0, 1.0, 1.0, 3),            # every coordinate kept and sent: only the codes compress
    (65_537, 2, 0, 1.0, 0.3, 3),
    (300_001, 3, 3, 0.03, 0.004, 5),
])
def test_composed_trajectories(ddef, oracle_mod, d, n, tau, rho, delta, steps):
    w = workloads.replace(workloads.get("C3", d=d, n=n), seed=2000 + d)
    g, o = pair(ddef, oracle_mod, w, tau, rho)
    k = oracle_mod.k_from_delta(delta, oracle_mod.k_from_delta(rho, d))
    for t in range(steps):
        g.grad(); o.grad()
        g.ef_compress(delta, w.lr); o.ef_compress(delta, w.lr)
        g.aggregate(); o.aggregate()
        g.apply_delayed(w.lr); o.apply_delayed()
        assert_same(g, o, n, (d, t))
        if t >= tau:
            assert len(g.get_message(0)[0]) == k
    g.close()


def test_ties_and_zero_blocks(ddef, oracle_mod):
    # loaded gradients with many equal magnitudes, +-0 and a stretch of zeros long enough to fill
    # whole blocks of the message: the tie rule and the zero-step rule
    d, n = 40_000, 2
    w = workloads.replace(workloads.get("C1", d=d, n=n), seed=77, noise_kind=0, noise_scale=0.0)
    g, o = pair(ddef, oracle_mod, w, 0, 1.0)
    rng = np.random.default_rng(8)
    for t in range(3):
        for i in range(n):
            v = rng.choice(np.array([0.0, -0.0, 1.0, -1.0, 2.5, 1e-42], dtype=F32), d, p=[0.6, 0.1, 0.1, 0.1, 0.05, 0.05])
            g.load_grad(i, v); o.load_grad(i, v)
        g.ef_compress(0.9, 1.0); o.ef_compress(0.9, 1.0)
        g.aggregate(); o.aggregate()
        g.apply_delayed(1.0); o.apply_delayed()
        assert_same(g, o, n, ("ties", t))
    g.close()


def test_switching_between_the_three_compressors(ddef, oracle_mod):
    w = workloads.get("C1", d=120_000, n=3)
    g, o = pair(ddef, oracle_mod, w, 1, 0.2)
    plan = [0, 0, 0, 2, 2, 0, 0, 1, 2, 0, 0, 0]
    for t, comp in enumerate(plan):
        g.set_compressor(comp); o.set_compressor(comp)
        delta = 0.1 if comp == 2 else 0.01
        g.step(delta, w.lr); o.step(delta, w.lr)
        assert_same(g, o, w.n, (t, comp), codes=comp == 2)
    g.close()


def test_growing_message_keeps_codes_in_step(ddef, oracle_mod):
    # delta changes from iteration to iteration, so the message rows and the code rows are reallocated
    w = workloads.get("C1", d=200_000, n=2)
    g, o = pair(ddef, oracle_mod, w, 0, 0.2)
    for t, delta in enumerate([0.01, 0.1, 0.5, 1.0, 0.02]):
        g.step(delta, w.lr); o.step(delta, w.lr)
        assert_same(g, o, w.n, (t, delta))
    g.close()


@pytest.mark.parametrize("compressor,percent", [(2, 0), (2, 60), (1, 0), (1, 95)])
def test_many_kept_coordinates_are_binned(ddef, oracle_mod, compressor, percent):
    # k1 >= 2^20 kept coordinates per worker: the bits are set through the region buckets; with
    # buckets sized below their expected fill a good part of them goes the bit-by-bit way instead
    d, n = 6_000_000, 2
    w = workloads.replace(workloads.get("C1", d=d, n=n), seed=91)
    g, o = pair(ddef, oracle_mod, w, 0, 0.2)
    g.set_compressor(compressor); o.set_compressor(compressor)
    g.set_option(ddef.OPT_RANDK_BUCKET_PERCENT, percent)
    delta = 0.1 if compressor == 2 else 0.2
    for t in range(3):
        g.step(delta, w.lr); o.step(delta, w.lr)
        assert_same(g, o, n, (compressor, percent, t), codes=compressor == 2)
    g.close()


@pytest.mark.parametrize("option", ["fuse", "prefetch", "noniid"])
def test_composed_under_the_library_options(ddef, oracle_mod, option):
    # the gradient options fall back to a stored gradient under this compressor; heterogeneous
    # optima only change the gradient: the trajectory must not depend on any of them
    w = workloads.replace(workloads.get("C3", d=150_001, n=3), seed=404)
    g, o = pair(ddef, oracle_mod, w, 2, 0.2)
    if option == "fuse":
        g.set_option(ddef.OPT_FUSE_GRAD, 1)
    elif option == "prefetch":
        g.set_option(ddef.OPT_PREFETCH_GRAD, 1)
    else:
        g.set_heterogeneity(0.4); o.set_heterogeneity(0.4)
    for t in range(7):
        g.step(0.1, w.lr); o.step(0.1, w.lr)
        assert_same(g, o, w.n, (option, t))
    g.close()


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_bounded_recording_and_its_repeat(ddef, oracle_mod, mode):
    # 0: every kept entry is recorded; 1: only those above the sampled bound; 2: the bound is placed
    # too high on purpose, every iteration is repeated without it.  Same results in all three.
    w = workloads.replace(workloads.get("C3", d=400_003, n=3), seed=515)
    g, o = pair(ddef, oracle_mod, w, 1, 0.2)
    g.set_option(ddef.OPT_COMPOSED_BOUND, mode)
    for t in range(6):
        g.step(0.1, w.lr); o.step(0.1, w.lr)
        assert_same(g, o, w.n, (mode, t))
    repeats = g.full_select_count()
    assert repeats == (5 * w.n if mode == 2 else 0)          # five non-empty iterations
    g.close()


def test_seeded_sweep_of_small_shapes(ddef, oracle_mod):
    """Forty seeded configurations with d from 1 to a few tens of thousands, the two ratios, tau and
    the compressor changing in mid-run (Random-k and the composed one share the marking pass)."""
    rng = np.random.default_rng(20250718)
    for case in range(40):
        d = int(rng.choice([1, 2, 5, 63, 64, 255, 257, 1023, 1025, 4096, 4097, 9000, 20011, 70001]))
        n = int(rng.integers(1, 5))
        tau_max = int(rng.integers(0, 3))
        kind = int(rng.integers(0, 3))
        w = workloads.replace(workloads.get("C1", d=d, n=n), seed=3000 + case, noise_kind=kind,
                              noise_scale=float(rng.choice([0.05, 0.5])) if kind else 0.0)
        lam, xstar, x0 = workloads.make_problem(w)
        g = ddef.Context(d, n, tau_max)
        o = oracle_mod.Oracle(d, n, tau_max, threads=2)
        for h in (g, o):
            h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        what = dict(case=case, d=d, n=n, tau_max=tau_max, kind=kind)
        for t in range(int(rng.integers(3, 8))):
            tau = int(rng.integers(0, tau_max + 1))
            comp = int(rng.choice([2, 2, 2, 1, 0]))
            rho = float(rng.choice([0.01, 0.2, 0.5, 1.0]))
            delta = float(rng.choice([0.003, 0.05, 0.1, 0.5, 1.0]))
            for h in (g, o):
                h.set_tau(tau); h.set_compressor(comp); h.set_composed(rho)
            g.step(delta, 0.05); o.step(delta, 0.05)
            assert_same(g, o, n, (what, t, comp, rho, delta), codes=comp == 2)
        g.close()
        o.close()


def test_argument_and_state_checks(ddef):
    c = ddef.Context(1000, 1, 0)
    one = np.ones(1000, dtype=F32)
    c.set_problem(one, one, one, 0, 0, 0.0)
    assert c.raw("set_composed", 0.0) == ddef.EINVAL
    assert c.raw("set_composed", 1.5) == ddef.EINVAL
    assert c.raw("set_composed", float("nan")) == ddef.EINVAL
    import ctypes as C
    k = C.c_uint64()
    assert c.raw("get_message_codes", 0, None, None, C.byref(k)) == ddef.ESTATE      # Top-k is selected
    c.set_compressor(ddef.COMPRESSOR_COMPOSED)
    assert c.raw("get_message_codes", 1, None, None, C.byref(k)) == ddef.EINVAL
    assert c.raw("get_message_codes", 0, None, None, None) == ddef.EINVAL
    c.grad()
    assert c.raw("set_composed", 0.5) == ddef.ESTATE
    c.ef_compress(0.1, 0.05); c.aggregate(); c.apply_delayed(0.05)
    idx, val = c.get_message(0)
    assert len(idx) == 20                   # ceil(0.1 * ceil(0.2 * 1000))
    codes, steps = c.get_message_codes(0)
    assert len(codes) == 10 and len(steps) == 1
    c.close()
    q = ddef.Context(1000, 1, 1, queue_form=True)
    assert q.raw("set_compressor", ddef.COMPRESSOR_COMPOSED) == ddef.EINVAL
    q.close()


def test_composed_c3_full_size(ddef, oracle_mod):
    # the paper's setting of this compressor (20 %, 10 %, tau = 1) on the C3 shape
    w = workloads.get("C3")
    lam, xstar, x0 = workloads.make_problem(w)
    g = ddef.Context(w.d, w.n, 1)
    o = oracle_mod.Oracle(w.d, w.n, 1, threads=w.n)
    for h in (g, o):
        h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        h.set_tau(1)
        h.set_compressor(2)
        h.set_composed(0.2)
    for t in range(3):
        g.step(0.1, w.lr)
        o.step(0.1, w.lr)
    assert_same(g, o, w.n, "C3 composed")
    g.close()
