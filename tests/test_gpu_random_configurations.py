"""Seeded random configurations of the whole step against the oracle, bit for bit: vector lengths
from 1 to a few million, 1 to 70 workers, all three compressors, snapshot ring and message queue,
(tau, delta) changing inside the run, every noise kind, heterogeneous optima, inputs with few
distinct values (ties at every threshold), and the library's options in random combinations
(fused or prefetched gradient, no filter, other candidate targets, the dense split's test modes,
the composed compressor's bound modes, undersized Random-k buckets)."""
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


def draw_case(rng, ddef):
    kind = str(rng.choice(["ring-topk", "ring-topk", "ring-topk", "ring-randk", "ring-composed", "queue-topk"]))
    d = int(10 ** rng.uniform(0, 6.5))
    if kind == "ring-composed":
        d = max(d, 64)
    n = int(rng.choice([1, 2, 3, 4, 5, 8, 16, 17, 24, 40, 70]))
    if d * n > 10_000_000:
        n = max(1, 10_000_000 // d)
    tau_max = int(rng.integers(0, 5))
    noise_kind = int(rng.integers(0, 3))
    zeta = float(rng.choice([0.0, 0.0, 0.3]))
    steps = int(rng.integers(3, 8)) + tau_max
    lr = float(rng.choice([0.05, 0.1, 0.01]))
    opts = {}
    if kind.startswith("ring"):
        if rng.random() < 0.25:
            opts[ddef.OPT_FUSE_GRAD] = 1
        elif rng.random() < 0.2 and tau_max >= 1:
            opts[ddef.OPT_PREFETCH_GRAD] = 1
        if rng.random() < 0.15:
            opts[ddef.OPT_FORCE_FULL_SELECT] = 1
        if rng.random() < 0.3:
            opts[ddef.OPT_CANDIDATE_SLACK_X16] = int(rng.choice([17, 24, 32, 64]))
        if rng.random() < 0.4:
            opts[ddef.OPT_DENSE_SPLIT] = int(rng.choice([0, 2, 3, 4]))
        if kind == "ring-composed" and rng.random() < 0.5:
            opts[ddef.OPT_COMPOSED_BOUND] = int(rng.choice([0, 2]))
        if kind == "ring-randk" and rng.random() < 0.3:
            opts[ddef.OPT_RANDK_BUCKET_PERCENT] = int(rng.choice([20, 100, 300]))
    w = workloads.replace(workloads.get("C1", d=d, n=n), seed=int(rng.integers(1, 2 ** 40)), noise_kind=noise_kind,
                          noise_scale=float(rng.choice([0.05, 0.5, 0.0 if noise_kind == 0 else 1.0])))
    few_values = rng.random() < 0.2
    sched = []
    tau = int(rng.integers(0, tau_max + 1))
    delta = float(10 ** rng.uniform(-3.5, 0))
    for _ in range(steps):
        if rng.random() < 0.25:
            tau = int(rng.integers(0, tau_max + 1))
        if rng.random() < 0.25:
            delta = float(min(1.0, 10 ** rng.uniform(-3.5, 0.05)))
        sched.append((tau, delta))
    rho = float(rng.choice([0.2, 0.5, 0.05]))
    return kind, w, tau_max, zeta, lr, opts, few_values, sched, rho


@pytest.mark.parametrize("seed", [101, 102, 103, 104])
def test_random_configurations_match_the_oracle(ddef, oracle_mod, seed):
    rng = np.random.default_rng(seed)
    for case in range(25):
        kind, w, tau_max, zeta, lr, opts, few_values, sched, rho = draw_case(rng, ddef)
        what = (seed, case, kind, w.d, w.n, tau_max, w.noise_kind, zeta, lr, opts, rho, sched)
        print("configuration", what, flush=True)
        lam, xstar, x0 = workloads.make_problem(w)
        if few_values:
            x0 = (np.round(x0 * 2) / 2).astype(F32)
            xstar = (np.round(xstar * 2) / 2).astype(F32)
            lam = np.full(w.d, 0.5, dtype=F32)
        queue = kind == "queue-topk"
        g = ddef.Context(w.d, w.n, tau_max, queue_form=queue)
        o = (oracle_mod.QueueOracle(w.d, w.n, sched[0][0]) if queue
             else oracle_mod.Oracle(w.d, w.n, tau_max, threads=min(w.n, 8)))
        for h in (g, o):
            h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
            if zeta:
                h.set_heterogeneity(zeta)
        comp = {"topk": 0, "randk": 1, "composed": 2}[kind.split("-")[1]]
        if not queue:
            for h in (g, o):
                h.set_compressor(comp)
                h.set_composed(rho)
            for option, value in opts.items():
                g.set_option(option, value)
        for t, (tau, delta) in enumerate(sched):
            for h in (g, o):
                h.set_tau(tau)
                h.step(delta, lr)
            for i in sorted({0, w.n - 1, int(rng.integers(0, w.n))}):
                gi, gv = g.get_message(i)
                oi, ov = o.get_message(i)
                assert np.array_equal(gi, oi), ("indices", t, i, what)
                assert np.array_equal(bits(gv), bits(ov)), ("values", t, i, what)
                assert np.array_equal(bits(g.get_error(i)), bits(o.get_error(i))), ("error buffer", t, i, what)
                if comp != 1 and not queue and len(oi):
                    assert g.get_threshold(i) == o.get_threshold(i), ("threshold", t, i, what)
            assert np.array_equal(bits(g.get_update()), bits(o.get_update())), ("update", t, what)
            assert np.array_equal(bits(g.get_model()), bits(o.get_model())), ("model", t, what)
        g.close()
        o.close()
