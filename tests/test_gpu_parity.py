"""GPU parity: the HIP path, called through the C-ABI, against the CPU oracle on the same
seeded inputs.  Bar: selected indices, message values, error buffers and gradients bit-exact;
the aggregated update and the model bit-exact too (the GPU sums in worker order like the
oracle), asserted at the stated tolerance of 1e-6 relative and reported when not exact."""
import numpy as np
import pytest

from paper_2507_17346_amd import workloads

pytestmark = pytest.mark.gpu

F32 = np.float32


def bits(a):
    return np.asarray(a, dtype=F32).view(np.uint32)


def rel_err(a, b):
    """max |a-b| / max(|b|, 1e-3 * ||b||_inf): the floor keeps exact zeros of b comparable."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    floor = 1e-3 * max(np.abs(b).max(), 1e-30)
    return float((np.abs(a - b) / np.maximum(np.abs(b), floor)).max())


@pytest.fixture(scope="module")
def ddef():
    from paper_2507_17346_amd import binding
    binding.load()
    return binding


def make_pair(ddef, oracle_mod, w, tau=None, tau_max=None, threads=4):
    lam, xstar, x0 = workloads.make_problem(w)
    tau = w.tau if tau is None else tau
    tau_max = max(tau, w.tau_max) if tau_max is None else tau_max
    g = ddef.Context(w.d, w.n, tau_max)
    g.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    g.set_tau(tau)
    o = oracle_mod.Oracle(w.d, w.n, tau_max, threads=threads)
    o.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    o.set_tau(tau)
    return g, o, (lam, xstar, x0)


def assert_step_state_equal(g, o, n, check_grad=True, what=""):
    for i in range(n):
        gi, gv = g.get_message(i)
        oi, ov = o.get_message(i)
        assert len(gi) == len(oi), (what, i)
        assert np.array_equal(gi, oi), (what, "indices", i)
        assert np.array_equal(bits(gv), bits(ov)), (what, "values", i)
        assert np.array_equal(bits(g.get_error(i)), bits(o.get_error(i))), (what, "error buffer", i)
        if len(oi):
            assert g.get_threshold(i) == o.get_threshold(i), (what, "threshold", i)
            if check_grad:
                assert np.array_equal(bits(g.get_grad(i)), bits(o.get_grad(i))), (what, "gradient", i)


def assert_model_equal(g, o, what=""):
    gu, ou = g.get_update(), o.get_update()
    gx, ox = g.get_model(), o.get_model()
    assert rel_err(gu, ou) <= 1e-6, what
    assert rel_err(gx, ox) <= 1e-6, what
    # worker-ordered summation on both sides: expected to agree to the bit
    assert np.array_equal(bits(gu), bits(ou)), what
    assert np.array_equal(bits(gx), bits(ox)), what


# ---- S0: gradient with counter-based noise -------------------------------------------------
@pytest.mark.parametrize("kind,scale", [(1, 0.1), (2, 0.05), (0, 0.0)])
@pytest.mark.parametrize("d", [1, 5, 4097, 300_001])
def test_gradient_bit_exact(ddef, oracle_mod, kind, scale, d):
    w = workloads.replace(workloads.get("C1", d=d, n=3), noise_kind=kind, noise_scale=scale, seed=0xABCDEF0123)
    g, o, _ = make_pair(ddef, oracle_mod, w, tau=0)
    for _ in range(2):
        g.grad()
        o.grad()
        for i in range(w.n):
            assert np.array_equal(bits(g.get_grad(i)), bits(o.get_grad(i))), (kind, d, i)
        g.ef_compress(0.5, 0.05); g.aggregate(); g.apply_delayed(0.05)
        o.ef_compress(0.5, 0.05); o.aggregate(); o.apply_delayed()
    g.close()


def test_gradient_noise_far_counters(ddef, oracle_mod):
    # step index beyond 2^32 is not reachable by stepping; large j and several workers are
    w = workloads.replace(workloads.get("C3", d=70_001, n=5), seed=(0xFEEDFACE << 32) | 0x1234)
    g, o, _ = make_pair(ddef, oracle_mod, w, tau=0)
    for _ in range(3):
        g.step(0.01, 0.05)
        o.step(0.01, 0.05)
    g.grad(); o.grad()
    for i in range(w.n):
        assert np.array_equal(bits(g.get_grad(i)), bits(o.get_grad(i)))
    g.close()


# ---- S1-S3: error feedback + Top-k on crafted inputs -----------------------------------------
KINDS = ["normal", "heavy", "few_values", "all_equal", "signed_zero", "denormal", "wide"]


@pytest.mark.parametrize("kind", KINDS)
@pytest.mark.parametrize("d", [1, 3, 1023, 4096, 4097, 20_000])
def test_compress_crafted_vectors(ddef, oracle_mod, kind, d):
    n = 2
    g = ddef.Context(d, n, 0)
    o = oracle_mod.Oracle(d, n, 0)
    zero = np.zeros(d, dtype=F32)
    for h in (g, o):
        h.set_problem(np.ones(d, dtype=F32), zero, zero, 1, 0, 0.0)
    ks = sorted({1, max(1, d // 1000), max(1, d // 7), max(1, d - 1), d})
    for step, k in enumerate(ks):
        delta = k / d if k < d else 1.0
        assert oracle_mod.k_from_delta(delta, d) == k == ddef.k_from_delta(delta, d)
        for i in range(n):
            v = workloads.random_vector(1000 * step + 10 * i + d, d, kind)
            g.load_grad(i, v)
            o.load_grad(i, v)
        g.ef_compress(delta, 1.0)
        o.ef_compress(delta, 1.0)
        assert_step_state_equal(g, o, n, check_grad=False, what=(kind, d, k))
        g.aggregate(); o.aggregate()
        g.apply_delayed(1.0); o.apply_delayed()
        assert_model_equal(g, o, what=(kind, d, k))
    g.close()


def test_compress_ties_across_chunks(ddef, oracle_mod):
    # the threshold group straddles several 4096-element chunks and only part of it is sent
    d, n = 40_000, 1
    v = np.full(d, 0.25, dtype=F32)
    v[::3] = -0.25
    v[5::1000] = 2.0
    g = ddef.Context(d, n, 0)
    o = oracle_mod.Oracle(d, n, 0)
    zero = np.zeros(d, dtype=F32)
    for h in (g, o):
        h.set_problem(np.ones(d, dtype=F32), zero, zero, 1, 0, 0.0)
    for k in [1, 39, 40, 41, 5000, 12_345, 39_999, 40_000]:
        g.load_grad(0, v); o.load_grad(0, v)
        g.ef_compress(k / d, 1.0); o.ef_compress(k / d, 1.0)
        assert_step_state_equal(g, o, n, check_grad=False, what=k)
        g.aggregate(); o.aggregate(); g.apply_delayed(1.0); o.apply_delayed()
    g.close()


# ---- whole trajectories, free running ----------------------------------------------------------
@pytest.mark.parametrize("name,d,n,tau,delta,steps", [
    ("C1", 50_000, 4, 2, 0.01, 12),
    ("C1", 9_999, 1, 0, 0.05, 8),
    ("C2", 200_003, 8, 4, 0.01, 10),
    ("C3", 150_001, 8, 3, 0.001, 9),
    ("C4", 131_072, 4, 1, 0.1, 6),
    ("C1", 4_096, 3, 5, 1.0, 9),
    ("C1", 9_001, 300, 1, 0.02, 5),        # more workers than one batch of the tile sum holds
    ("C1", 3, 2, 0, 0.5, 4),
])
def test_trajectory_free_running(ddef, oracle_mod, name, d, n, tau, delta, steps):
    w = workloads.get(name, d=d, n=n)
    g, o, _ = make_pair(ddef, oracle_mod, w, tau=tau)
    for t in range(steps):
        g.grad(); o.grad()
        g.ef_compress(delta, w.lr); o.ef_compress(delta, w.lr)
        assert_step_state_equal(g, o, n, check_grad=(t >= tau), what=(name, t))
        g.aggregate(); o.aggregate()
        g.apply_delayed(w.lr); o.apply_delayed()
        assert g.t == o.t == t + 1
        assert_model_equal(g, o, what=(name, t))
    g.close()


def test_c1_full_configuration(ddef, oracle_mod):
    w = workloads.get("C1")
    g, o, _ = make_pair(ddef, oracle_mod, w, threads=4)
    for t in range(w.steps):
        g.step(w.deltas[0], w.lr)
        o.step(w.deltas[0], w.lr)
        if t in (2, 3, 10, w.steps - 1):
            assert_step_state_equal(g, o, w.n, what=("C1", t))
            assert_model_equal(g, o, what=("C1", t))
    g.close()


def test_adaptive_schedule_changing_delta_and_tau(ddef, oracle_mod):
    # Algorithm 2: (delta, tau) re-chosen every E iterations.  Shrunk version of the adaptive
    # workload; the schedule comes from the library's DeCo on the seeded network trace.
    w = workloads.get("C5", d=120_000, n=4)
    w = workloads.replace(w, steps=40, adaptive_period=5)
    trace = workloads.network_trace(w)
    g, o, _ = make_pair(ddef, oracle_mod, w, tau=0, tau_max=w.tau_max)
    for t in range(w.steps):
        if t % w.adaptive_period == 0:
            p = t // w.adaptive_period
            tau, delta = ddef.deco(trace.v_g_bits, trace.bandwidth_bps[p], trace.latency_s[p], trace.t_comp_s)
            assert (tau, pytest.approx(delta, rel=1e-12)) == oracle_mod.deco(
                trace.v_g_bits, trace.bandwidth_bps[p], trace.latency_s[p], trace.t_comp_s)
            tau = int(np.clip(tau, *trace.tau_bounds))
            delta = float(np.clip(delta, *trace.delta_bounds))
            g.set_tau(tau); o.set_tau(tau)
        g.grad(); o.grad()
        g.ef_compress(delta, w.lr); o.ef_compress(delta, w.lr)
        assert_step_state_equal(g, o, w.n, check_grad=False, what=("C5", t))
        g.aggregate(); o.aggregate()
        g.apply_delayed(w.lr); o.apply_delayed()
        assert_model_equal(g, o, what=("C5", t))
    g.close()


def test_changing_k_keeps_the_candidate_filter(ddef, oracle_mod):
    """delta moves by factors of 3 to 10 in both directions (Algorithm 2 re-chooses it): the bound
    is re-placed for the new k from the tail the last selection measured, so the filter keeps
    carrying the selections; whatever search runs, the result equals the oracle's."""
    w = workloads.get("C3", d=2_000_000, n=2)
    g, o, _ = make_pair(ddef, oracle_mod, w, tau=0, tau_max=0, threads=2)
    schedule = [0.001] * 6 + [0.01] * 4 + [0.001] * 4 + [0.003] * 3 + [0.0005] * 3
    for t, delta in enumerate(schedule):
        g.step(delta, w.lr); o.step(delta, w.lr)
        assert_step_state_equal(g, o, w.n, check_grad=False, what=("k change", t, delta))
        assert_model_equal(g, o, what=("k change", t))
    # neither the first iterations nor the changes of k need a whole-row search
    assert g.full_select_count() == 0, g.full_select_count()
    g.close()


# ---- checkpoint hooks and teacher forcing ---------------------------------------------------------
def test_teacher_forced_step(ddef, oracle_mod):
    w = workloads.get("C1", d=30_000, n=2)
    g, o, _ = make_pair(ddef, oracle_mod, w, tau=0)
    rng = np.random.default_rng(5)
    for t in range(3):
        x = rng.standard_normal(w.d, dtype=F32)
        g.set_model(x); o.set_model(x)
        for i in range(w.n):
            e = (rng.standard_normal(w.d, dtype=F32) * F32(0.01))
            g.set_error(i, e); o.set_error(i, e)
        g.step(0.02, w.lr); o.step(0.02, w.lr)
        assert_step_state_equal(g, o, w.n, what=t)
        assert_model_equal(g, o, what=t)
    g.close()


# ---- boundary behaviour: call order and argument checks ---------------------------------------------
def test_state_machine_and_errors(ddef):
    import ctypes as C
    lib = ddef.load()
    h = C.c_void_p()
    assert lib.ddef_init(0, 1, 0, C.byref(h)) == ddef.EINVAL
    assert lib.ddef_init(10, 0, 0, C.byref(h)) == ddef.EINVAL
    assert lib.ddef_init(1 << 32, 1, 0, C.byref(h)) == ddef.EINVAL
    assert lib.ddef_init(10, 1, 0, None) == ddef.EINVAL
    d = 1000
    c = ddef.Context(d, 2, 3)
    one = np.ones(d, dtype=F32)
    assert c.raw("grad") == ddef.ESTATE                       # no problem yet
    c.set_problem(one, one, one, 0, 1, 0.1)
    assert c.raw("set_tau", 4) == ddef.EINVAL
    assert c.raw("ef_compress", C.c_double(0.1), C.c_float(0.1)) == ddef.ESTATE
    assert c.raw("aggregate") == ddef.ESTATE
    assert c.raw("apply_delayed", C.c_float(0.1)) == ddef.ESTATE
    c.set_tau(0)
    c.grad()
    assert c.raw("grad") == ddef.ESTATE
    assert c.raw("set_tau", 1) == ddef.ESTATE
    for bad in (0.0, -0.5, 1.5, float("nan")):
        assert c.raw("ef_compress", C.c_double(bad), C.c_float(0.1)) == ddef.EINVAL
    assert c.raw("ef_compress", C.c_double(0.1), C.c_float(float("inf"))) == ddef.EINVAL
    c.ef_compress(0.1, 0.05)
    assert c.raw("apply_delayed", C.c_float(0.05)) == ddef.ESTATE
    c.aggregate()
    assert c.raw("apply_delayed", C.c_float(0.06)) == ddef.EINVAL      # not this step's stepsize
    c.apply_delayed(0.05)
    assert c.t == 1
    assert c.raw("get_error", 2, one.ctypes.data_as(C.POINTER(C.c_float))) == ddef.EINVAL
    assert c.raw("load_grad", 0, None) == ddef.EINVAL
    c.close()


def test_empty_iterations_before_tau(ddef):
    d, tau = 5000, 3
    w = workloads.get("C1", d=d, n=2)
    lam, xstar, x0 = workloads.make_problem(w)
    c = ddef.Context(d, 2, tau)
    c.set_problem(lam, xstar, x0, 0, 1, 0.1)
    for t in range(tau):
        c.step(0.1, 0.05)
        assert len(c.get_message(0)[0]) == 0
        assert np.array_equal(bits(c.get_model()), bits(x0))
        assert np.all(bits(c.get_update()) == 0)
        assert np.all(bits(c.get_error(1)) == 0)
    c.step(0.1, 0.05)
    assert len(c.get_message(0)[0]) == 500
    assert not np.array_equal(bits(c.get_model()), bits(x0))
    c.close()


# ---- candidate filter: used in the steady state, abandoned safely when its bound is off -------------
def test_filter_path_is_used_and_matches_full_search(ddef, oracle_mod):
    w = workloads.get("C3", d=400_000, n=4)
    lam, xstar, x0 = workloads.make_problem(w)
    a = ddef.Context(w.d, w.n, 0)
    b = ddef.Context(w.d, w.n, 0)
    b.set_option(ddef.OPT_FORCE_FULL_SELECT, 1)
    o = oracle_mod.Oracle(w.d, w.n, 0, threads=4)
    for h in (a, b, o):
        h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        h.set_tau(0)
    steps = 12
    for t in range(steps):
        a.step(0.002, w.lr); b.step(0.002, w.lr); o.step(0.002, w.lr)
        assert_step_state_equal(a, o, w.n, what=("filter", t))
        assert_step_state_equal(b, o, w.n, what=("full", t))
        assert_model_equal(a, o, what=("filter", t))
    assert b.full_select_count() == steps * w.n
    # the first two bounds come from samples of p, the later ones from the selections before them:
    # the filter carries every selection
    assert a.full_select_count() == 0, a.full_select_count()
    a.close(); b.close()


def test_filter_bound_too_high_and_too_low_fall_back(ddef, oracle_mod):
    d, n = 300_000, 2
    g = ddef.Context(d, n, 0)
    o = oracle_mod.Oracle(d, n, 0)
    zero = np.zeros(d, dtype=F32)
    for h in (g, o):
        h.set_problem(np.ones(d, dtype=F32), zero, zero, 1, 0, 0.0)
    delta = 0.004
    scales = [1.0, 1.0, 1e-3, 1e-3, 1e3, 1e3, 1.0, 0.5, 2.0, 1.0, 1.0, 1.0, 0.85, 0.85]
    fulls = []
    for step, sc in enumerate(scales):
        for i in range(n):
            v = workloads.random_vector(77 * step + i, d, "normal") * F32(sc)
            g.set_error(i, zero); o.set_error(i, zero)
            g.load_grad(i, v); o.load_grad(i, v)
        g.ef_compress(delta, 1.0); o.ef_compress(delta, 1.0)
        assert_step_state_equal(g, o, n, check_grad=False, what=("scale", step, sc))
        g.aggregate(); o.aggregate(); g.apply_delayed(1.0); o.apply_delayed()
        assert_model_equal(g, o, what=("scale", step))
        fulls.append(g.full_select_count())
    # steps 0 and 1 place their bound from a sample of p and need no row search.  step 2: magnitudes
    # dropped 1000x -> too few candidates.  step 4: rose 10^6x -> candidate buffer overflows.  Each of
    # these must have taken the whole-row search, and the step after it must not.
    assert fulls[0] == 0 and fulls[1] == 0
    assert fulls[2] == n and fulls[3] == n
    assert fulls[4] == 2 * n and fulls[5] == 2 * n
    assert fulls[11] == fulls[10] and fulls[12] == fulls[11] + n
    g.close()


def test_filter_with_ties_at_the_threshold(ddef, oracle_mod):
    d, n = 200_000, 1
    g = ddef.Context(d, n, 0)
    o = oracle_mod.Oracle(d, n, 0)
    zero = np.zeros(d, dtype=F32)
    for h in (g, o):
        h.set_problem(np.ones(d, dtype=F32), zero, zero, 1, 0, 0.0)
    rng = np.random.default_rng(3)
    for step in range(6):
        # few distinct magnitudes: the threshold group is large and only partly sent
        v = (rng.integers(0, 40, size=d).astype(F32) * F32(0.125)) * rng.choice([-1, 1], size=d).astype(F32)
        g.set_error(0, zero); o.set_error(0, zero)
        g.load_grad(0, v); o.load_grad(0, v)
        delta = [0.01, 0.01, 0.012, 0.03, 0.03, 0.005][step]
        g.ef_compress(delta, 1.0); o.ef_compress(delta, 1.0)
        assert_step_state_equal(g, o, n, check_grad=False, what=("ties", step))
        g.aggregate(); o.aggregate(); g.apply_delayed(1.0); o.apply_delayed()
    assert g.full_select_count() < 6
    g.close()


def test_non_finite_values_are_reported(ddef):
    d = 10_000
    c = ddef.Context(d, 2, 0)
    one = np.ones(d, dtype=F32)
    c.set_problem(one, one, one, 0, 0, 0.0)
    c.step(0.1, 0.05)
    assert c.raw("sync") == ddef.OK
    g = np.zeros(d, dtype=F32)
    g[1234] = np.inf
    c.load_grad(0, np.zeros(d, dtype=F32))
    c.load_grad(1, g)
    c.ef_compress(0.1, 0.05)
    assert c.raw("sync") == ddef.ENONFINITE
    assert c.raw("aggregate") == ddef.ENONFINITE          # refused until a fresh problem is set
    c.set_problem(one, one, one, 0, 0, 0.0)
    c.step(0.1, 0.05)
    assert c.raw("sync") == ddef.OK
    c.close()


# ---- gradient prefetch on a second stream: same results ------------------------------------------
@pytest.mark.parametrize("tau", [0, 1, 3])
def test_prefetched_gradient_gives_identical_trajectories(ddef, oracle_mod, tau):
    w = workloads.get("C3", d=300_000, n=4)
    lam, xstar, x0 = workloads.make_problem(w)
    g = ddef.Context(w.d, w.n, 4)
    g.set_option(ddef.OPT_PREFETCH_GRAD, 1)
    o = oracle_mod.Oracle(w.d, w.n, 4, threads=4)
    for h in (g, o):
        h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        h.set_tau(tau)
    rng = np.random.default_rng(8)
    for t in range(14):
        if t == 6:                                  # staleness changes: a prefetched gradient is stale
            g.set_tau(min(tau + 1, 4)); o.set_tau(min(tau + 1, 4))
        if t == 9:                                  # so it is after the model was overwritten
            x = rng.standard_normal(w.d, dtype=F32)
            g.set_model(x); o.set_model(x)
        if t == 11:
            g.set_option(ddef.OPT_PREFETCH_GRAD, 0)
        g.grad(); o.grad()
        if t == 4:                                  # test hook on top of a prefetched gradient
            v = rng.standard_normal(w.d, dtype=F32)
            g.load_grad(1, v); o.load_grad(1, v)
        g.ef_compress(0.004, w.lr); o.ef_compress(0.004, w.lr)
        assert_step_state_equal(g, o, w.n, check_grad=(t >= 4), what=("prefetch", tau, t))
        g.aggregate(); o.aggregate()
        g.apply_delayed(w.lr); o.apply_delayed()
        assert_model_equal(g, o, what=("prefetch", tau, t))
    g.close()


# ---- gradient generated inside the accumulate pass: same results --------------------------------
@pytest.mark.parametrize("name,d,n,tau,delta", [("C3", 200_001, 4, 2, 0.002), ("C1", 50_000, 3, 0, 0.01),
                                                ("C2", 150_000, 8, 1, 0.01),
                                                ("C3", 300_001, 3, 1, 0.1),       # sampled bound every iteration
                                                ("C1", 70_000, 2, 3, 0.4)])
def test_fused_gradient_gives_identical_trajectories(ddef, oracle_mod, name, d, n, tau, delta):
    w = workloads.get(name, d=d, n=n)
    lam, xstar, x0 = workloads.make_problem(w)
    g = ddef.Context(w.d, w.n, max(tau, 1))
    g.set_option(ddef.OPT_FUSE_GRAD, 1)
    o = oracle_mod.Oracle(w.d, w.n, max(tau, 1), threads=4)
    for h in (g, o):
        h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        h.set_tau(tau)
    rng = np.random.default_rng(9)
    for t in range(tau + 9):
        if t == tau + 5:                               # Random-k reads a stored gradient: falls back
            g.set_compressor(1); o.set_compressor(1)
        if t == tau + 6:
            g.set_compressor(0); o.set_compressor(0)
        g.grad(); o.grad()
        if t == tau + 3:                               # the test hook needs the gradient in memory
            v = rng.standard_normal(w.d, dtype=F32)
            g.load_grad(0, v); o.load_grad(0, v)
        g.ef_compress(delta, w.lr); o.ef_compress(delta, w.lr)
        # in this mode the gradient can be fetched until the iteration is applied
        assert_step_state_equal(g, o, w.n, check_grad=(t >= tau), what=("fused", name, t))
        g.aggregate(); o.aggregate()
        g.apply_delayed(w.lr); o.apply_delayed()
        assert_model_equal(g, o, what=("fused", name, t))
    import ctypes as C
    buf = np.empty(w.d, dtype=F32)
    assert g.raw("get_grad", 0, buf.ctypes.data_as(C.POINTER(C.c_float))) == ddef.ESTATE
    g.close()


# ---- non-IID workers: per-worker optima --------------------------------------------------------
@pytest.mark.parametrize("fuse", [0, 1])
def test_heterogeneous_objectives(ddef, oracle_mod, fuse):
    w = workloads.get("C1", d=120_001, n=4)
    lam, xstar, x0 = workloads.make_problem(w)
    g = ddef.Context(w.d, w.n, 2)
    g.set_option(ddef.OPT_FUSE_GRAD, fuse)
    o = oracle_mod.Oracle(w.d, w.n, 2, threads=4)
    for h in (g, o):
        h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        h.set_tau(1)
        h.set_heterogeneity(0.4)
    for t in range(8):
        if t == 5:
            g.set_heterogeneity(0.0); o.set_heterogeneity(0.0)
        g.grad(); o.grad()
        g.ef_compress(0.01, w.lr); o.ef_compress(0.01, w.lr)
        assert_step_state_equal(g, o, w.n, check_grad=(t >= 1), what=("non-iid", fuse, t))
        g.aggregate(); o.aggregate()
        g.apply_delayed(w.lr); o.apply_delayed()
        assert_model_equal(g, o, what=("non-iid", fuse, t))
    g.close()


# ---- seeded sweep over small shapes ---------------------------------------------------------------
def test_seeded_sweep_of_small_shapes(ddef, oracle_mod):
    """Forty seeded configurations with d from 1 to a few thousand (ragged quads, groups, chunks and
    tiles), every noise kind, both server states, tau and delta changing in mid-run."""
    rng = np.random.default_rng(20250717)
    for case in range(40):
        d = int(rng.choice([1, 2, 3, 5, 63, 64, 255, 256, 257, 1023, 1025, 4095, 4096, 4097, 5000, 9000, 20011]))
        n = int(rng.integers(1, 6))
        tau_max = int(rng.integers(0, 4))
        kind = int(rng.integers(0, 3))
        queue = bool(rng.integers(0, 2))
        w = workloads.replace(workloads.get("C1", d=d, n=n), seed=1000 + case, noise_kind=kind,
                              noise_scale=float(rng.choice([0.0, 0.05, 0.5])) if kind else 0.0)
        lam, xstar, x0 = workloads.make_problem(w)
        g = ddef.Context(d, n, tau_max, queue_form=queue)
        o = oracle_mod.QueueOracle(d, n, tau_max) if queue else oracle_mod.Oracle(d, n, tau_max)
        for h in (g, o):
            h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        what = dict(case=case, d=d, n=n, tau_max=tau_max, kind=kind, queue=queue)
        for t in range(int(rng.integers(3, 9))):
            tau = int(rng.integers(0, tau_max + 1))
            delta = float(rng.choice([1e-4, 0.003, 0.01, 0.1, 0.5, 1.0]))
            lr = float(rng.choice([0.05, 0.3]))
            g.set_tau(tau); o.set_tau(tau)
            g.step(delta, lr); o.step(delta, lr)
            for i in range(n):
                gi, gv = g.get_message(i)
                oi, ov = o.get_message(i)
                assert np.array_equal(gi, oi), (what, t, i)
                assert np.array_equal(bits(gv), bits(ov)), (what, t, i)
                assert np.array_equal(bits(g.get_error(i)), bits(o.get_error(i))), (what, t, i)
            assert np.array_equal(bits(g.get_update()), bits(o.get_update())), (what, t)
            assert np.array_equal(bits(g.get_model()), bits(o.get_model())), (what, t)
        g.close()
        o.close()


# ---- checkpoint and resume -------------------------------------------------------------------------
@pytest.mark.parametrize("tau,graph", [(0, 0), (3, 0), (2, 1)])
def test_checkpoint_and_resume_continue_bit_for_bit(ddef, oracle_mod, tau, graph):
    w = workloads.get("C3", d=120_011, n=3)
    lam, xstar, x0 = workloads.make_problem(w)

    def fresh():
        c = ddef.Context(w.d, w.n, tau + 1)
        c.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        c.set_tau(tau)
        c.set_option(ddef.OPT_GRAPH, graph)
        return c

    a = fresh()
    o = oracle_mod.Oracle(w.d, w.n, tau + 1, threads=3)
    o.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    o.set_tau(tau)
    for t in range(9):
        a.step(0.004, w.lr); o.step(0.004, w.lr)
    # checkpoint: t, every snapshot still in the ring, every error buffer
    t_saved = a.t
    snaps = [a.get_snapshot(age) for age in range(min(t_saved, tau + 1) + 1)]
    errs = [a.get_error(i) for i in range(w.n)]
    assert a.raw("get_snapshot", tau + 2, snaps[0].ctypes.data_as(ddef._f32p)) == ddef.EINVAL
    a.close()
    # resume in a new context
    b = fresh()
    b.set_step_index(t_saved)
    for age, x in enumerate(snaps):
        b.set_snapshot(age, x)
    for i, e in enumerate(errs):
        b.set_error(i, e)
    for t in range(7):
        b.step(0.004, w.lr); o.step(0.004, w.lr)
        assert_step_state_equal(b, o, w.n, check_grad=False, what=("resumed", tau, t))
        assert_model_equal(b, o, what=("resumed", tau, t))
    assert b.t == t_saved + 7
    b.close()
    q = ddef.Context(1000, 2, 1, queue_form=True)
    assert q.raw("set_step_index", 3) == ddef.ESTATE
    q.close()


# --- dense messages: candidates sure to be sent bypass the selection ----------------------------
@pytest.mark.parametrize("mode", [1, 2, 3, 4, 0])
@pytest.mark.parametrize("d,n,delta", [(300_017, 3, 0.1), (70_001, 2, 0.3), (1_200_003, 4, 0.04),
                                       (40_009, 37, 0.07)])     # more workers than one round of run descriptors
def test_dense_messages_sure_and_band_split(ddef, oracle_mod, mode, d, n, delta):
    """Messages dense enough for the filter bound to come from a sample of p in every iteration
    (k/d > 1/32): candidates a margin above the expected threshold are recorded once and go to the
    aggregation as runs, the band around the threshold goes through the selection.  Messages (put
    together by the getter), thresholds, error buffers, update and model against the oracle; the test
    modes put the line where about half, none or all of the selections must fall back to their rows."""
    w = workloads.get("C1", d=d, n=n)
    w = workloads.replace(w, seed=900 + mode, tau=1, tau_max=1)
    lam, xstar, x0 = workloads.make_problem(w)
    g = ddef.Context(w.d, w.n, w.tau_max)
    o = oracle_mod.Oracle(w.d, w.n, w.tau_max, threads=w.n)
    for h in (g, o):
        h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        h.set_tau(w.tau)
    g.set_option(ddef.OPT_DENSE_SPLIT, mode)
    steps = 7
    for t in range(steps):
        g.step(delta, w.lr)
        o.step(delta, w.lr)
        assert_step_state_equal(g, o, w.n, what=("split", mode, t))
        assert np.array_equal(bits(g.get_update()), bits(o.get_update())), ("split update", mode, t)
        assert_model_equal(g, o, what=("split", mode, t))
    fell_back = g.full_select_count()
    real = (steps - w.tau) * w.n
    if mode in (0, 1, 3):
        assert fell_back == 0, fell_back
    if mode == 4:
        assert fell_back == real
    if mode == 2 and d > 2 ** 20:          # (a shorter row is sampled whole: the expected threshold is the true one)
        assert 0 < fell_back < real
    g.close()
    o.close()
