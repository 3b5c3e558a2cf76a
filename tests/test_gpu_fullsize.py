"""GPU parity at the workloads' full sizes, in the launch configuration bench.py times.

C2 and C3 are compared with the oracle element by element for every worker (the oracle needs a
few seconds per iteration with one thread per worker).  C4 (d = 1.3e9, n*d > 2^32): the oracle's
step runs whole for one worker (about a minute per iteration; all four would take four times the
memory and no less time) over one iteration per delta of the sweep, and its message, threshold
and error buffer are compared element by element; on top of that every watched worker's selection
is checked through properties that hold at any size (count, order, threshold dominance, tie rule,
EF identity) and gradients and error-feedback values on sampled coordinates that the oracle
computes one by one.
"""
import functools

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


def run_pair(ddef, oracle_mod, w, real_steps, delta):
    lam, xstar, x0 = workloads.make_problem(w)
    g = ddef.Context(w.d, w.n, w.tau_max)
    o = oracle_mod.Oracle(w.d, w.n, w.tau_max, threads=w.n)
    for h in (g, o):
        h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        h.set_tau(w.tau)
    for t in range(w.tau + real_steps):
        g.step(delta, w.lr)
        o.step(delta, w.lr)
        if t >= w.tau:
            # indices and thresholds of every worker at every iteration (cheap to fetch)
            for i in range(w.n):
                gi, gv = g.get_message(i)
                oi, ov = o.get_message(i)
                assert np.array_equal(gi, oi), (w.name, t, i)
                assert np.array_equal(bits(gv), bits(ov)), (w.name, t, i)
                assert g.get_threshold(i) == o.get_threshold(i)
    for i in range(w.n):
        assert np.array_equal(bits(g.get_error(i)), bits(o.get_error(i))), (w.name, "error buffer", i)
        assert np.array_equal(bits(g.get_grad(i)), bits(o.get_grad(i))), (w.name, "gradient", i)
    gu, ou = g.get_update(), o.get_update()
    gx, ox = g.get_model(), o.get_model()
    scale = np.abs(ox).max()
    assert np.abs(gx.astype(np.float64) - ox).max() <= 1e-6 * scale
    assert np.array_equal(bits(gu), bits(ou)) and np.array_equal(bits(gx), bits(ox))
    used_filter = w.n * real_steps - g.full_select_count()
    g.close()
    o.close()
    return used_filter


def test_c2_full_size(ddef, oracle_mod):
    w = workloads.get("C2")
    used = run_pair(ddef, oracle_mod, w, real_steps=6, delta=w.deltas[0])
    assert used >= 3 * w.n            # the candidate filter carried most selections


def test_c3_full_size_bench_configuration(ddef, oracle_mod):
    w = workloads.get("C3")
    used = run_pair(ddef, oracle_mod, w, real_steps=4, delta=w.deltas[0])
    assert used >= w.n                # at least the last iterations ran through the filter


@pytest.mark.parametrize("periods", [range(0, 5), range(5, 10)], ids=["periods 0-4", "periods 5-9"])
def test_c5_full_size_across_changes_of_tau_and_delta(ddef, oracle_mod, periods):
    """The adaptive workload at its real shape (d = 124e6, n = 16, ring of 17 snapshots) against the
    oracle over all ten periods of its DeCo schedule, the first two real iterations of each, in two
    runs of five periods (each from x_0, so that neither run is silent for minutes): tau rises
    (6 -> 9), falls (9 -> 2), reaches the ring's full depth (16), goes to 15; and 16, 6, 10, 7, 14
    in the second run, while delta moves between 0.0006 and 0.036 -- sparse messages whose filter
    bound follows the last thresholds, messages dense enough for a bound sampled in every iteration
    (delta = 0.0044 ... 0.0105), and dense ones whose sure candidates bypass the selection
    (delta = 0.036 > 1/32).  Every change re-places the filter bound and changes the length of the
    messages."""
    w = workloads.get("C5")
    trace = workloads.network_trace(w)
    whole = []
    for p in range(len(trace.bandwidth_bps)):
        tau, delta = ddef.deco(trace.v_g_bits, trace.bandwidth_bps[p], trace.latency_s[p], trace.t_comp_s)
        whole.append((int(np.clip(tau, *trace.tau_bounds)), float(np.clip(delta, *trace.delta_bounds))))
    taus = [tau for tau, _ in whole]
    assert len(whole) == 10 and taus[1] > taus[0] and taus[2] < taus[1] and max(taus) == w.tau_max
    assert any(ddef.k_from_delta(delta, w.d) * 32 > w.d for _, delta in whole)
    assert any(ddef.k_from_delta(delta, w.d) * w.n < 2 ** 23 for _, delta in whole)
    plan = [whole[p] for p in periods]
    lam, xstar, x0 = workloads.make_problem(w)
    g = ddef.Context(w.d, w.n, w.tau_max)
    o = oracle_mod.Oracle(w.d, w.n, w.tau_max, threads=w.n)
    for h in (g, o):
        h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    t = 0
    for period, (tau, delta) in zip(periods, plan):
        real = 0
        while real < 2:
            for h in (g, o):
                h.set_tau(tau)
                h.step(delta, w.lr)
            if t >= tau:
                real += 1
                print(f"C5 vs oracle: period {period} (tau {tau}, delta {delta:.5f}), iteration {t}", flush=True)
                for i in (0, 7, w.n - 1):
                    gi, gv = g.get_message(i)
                    oi, ov = o.get_message(i)
                    assert np.array_equal(gi, oi), ("C5", t, i)
                    assert np.array_equal(bits(gv), bits(ov)), ("C5", t, i)
                    assert g.get_threshold(i) == o.get_threshold(i), ("C5 threshold", t, i)
                assert np.array_equal(bits(g.get_model()), bits(o.get_model())), ("C5 model", t)
            t += 1
        for i in (0, w.n - 1):
            assert np.array_equal(bits(g.get_error(i)), bits(o.get_error(i))), ("C5 error buffer", period, i)
        assert np.array_equal(bits(g.get_update()), bits(o.get_update())), ("C5 update", period)
    assert g.full_select_count() < w.n          # (every change of k places its bound from a sample of p)
    g.close()
    o.close()


@functools.lru_cache(maxsize=1)
def c4_problem():
    w = workloads.get("C4")
    return (w,) + tuple(workloads.make_problem(w))


def test_c4_full_size_one_worker_against_the_oracle(ddef, oracle_mod):
    """C4 at its real shape on the GPU (d = 1.3e9, n = 4, tau = 4) against the oracle's step for
    worker 0, one iteration per delta of the sweep (0.01, 0.1, 0.001).  The oracle runs with one
    worker: a worker's messages and error buffer depend on the others only through the snapshot its
    gradient is taken at, and iterations tau .. 2 tau all take theirs at x_0 (the first update lands
    in x_{tau+1}), whatever the number of workers.  So the oracle, given only the seeded inputs,
    produces what worker 0 of the four must produce."""
    w, lam, xstar, x0 = c4_problem()
    g = ddef.Context(w.d, w.n, w.tau_max)
    o = oracle_mod.Oracle(w.d, 1, w.tau_max, threads=16)
    for h in (g, o):
        h.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        h.set_tau(w.tau)
    schedule = {w.tau: 0.01, w.tau + 1: 0.1, w.tau + 2: 0.001}
    for t in range(w.tau + 3):
        delta = schedule.get(t, 0.01)
        print(f"C4 vs oracle: iteration {t} delta {delta}", flush=True)
        g.step(delta, w.lr)
        o.step(delta, w.lr)
        if t < w.tau:
            continue
        gi, gv = g.get_message(0)
        oi, ov = o.get_message(0)
        assert len(gi) == ddef.k_from_delta(delta, w.d)
        assert np.array_equal(gi, oi), ("C4 indices", t)
        assert np.array_equal(bits(gv), bits(ov)), ("C4 values", t)
        assert g.get_threshold(0) == o.get_threshold(0), ("C4 threshold", t)
        del gi, gv, oi, ov
        ge = g.get_error(0)
        oe = o.get_error(0)
        assert np.array_equal(bits(ge), bits(oe)), ("C4 error buffer", t)
        del ge, oe
    assert np.array_equal(bits(g.get_grad(0)), bits(o.get_grad(0)))
    assert g.full_select_count() == 0          # every selection went through the sampled filter
    g.close()
    o.close()


def test_c4_full_size_properties_and_samples(ddef, oracle_mod):
    w, lam, xstar, x0 = c4_problem()
    g = ddef.Context(w.d, w.n, w.tau_max)
    g.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    g.set_tau(w.tau)
    # the workload sweeps delta; iterations tau .. 2*tau all take their gradient at x0
    schedule = {w.tau: 0.001, w.tau + 1: 0.001, w.tau + 2: 0.001, w.tau + 3: 0.01, w.tau + 4: 0.1}
    rng = np.random.default_rng(17)
    sample = np.unique(np.concatenate([rng.integers(0, w.d, size=4000),
                                       [0, 1, w.d - 1, w.d - 2, 2 ** 30, 2 ** 30 + 1]]))
    watched = (0, w.n - 1)                     # first and last worker: flat offsets beyond 2^32
    e_prev = {i: np.zeros(len(sample), dtype=F32) for i in watched}
    for t in range(2 * w.tau + 1):
        delta = schedule.get(t, 0.001)
        k = ddef.k_from_delta(delta, w.d)
        # the first real iteration searches the whole rows (the path without the candidate filter),
        # the others go through the filter, whose first bounds come from a sample of p
        g.set_option(ddef.OPT_FORCE_FULL_SELECT, 1 if t == w.tau else 0)
        g.grad()
        g.ef_compress(delta, w.lr)
        if t < w.tau:
            g.aggregate()
            g.apply_delayed(w.lr)
            continue
        for i in watched:
            idx, val = g.get_message(i)
            T, r = g.get_threshold(i)
            e_new = g.get_error(i)
            assert len(idx) == k
            assert np.all(np.diff(idx.astype(np.int64)) > 0) and int(idx[-1]) < w.d
            vkeys = bits(val) & np.uint32(0x7FFFFFFF)
            assert int(vkeys.min()) == T and int((vkeys == T).sum()) == r
            assert np.all(bits(e_new[idx]) == 0)             # sent entries leave the buffer
            ekeys = bits(e_new) & np.uint32(0x7FFFFFFF)
            assert int(ekeys.max()) <= T                      # nothing larger was left behind
            left = np.flatnonzero(ekeys == T)
            if len(left) and r:
                assert int(left.min()) > int(idx[vkeys == T].max())    # ties: lower indices sent first
            del ekeys, left
            # sampled coordinates: gradient and p = e + lr*g recomputed from the oracle's noise
            gs = g.get_grad(i)[sample]
            z = np.array([oracle_mod.noise_z(w.seed, t, i, int(j), w.noise_kind) for j in sample], dtype=F32)
            want_g = lam[sample] * (x0[sample] - xstar[sample]) + F32(w.noise_scale) * z
            assert np.array_equal(bits(gs), bits(want_g))
            p = e_prev[i] + F32(w.lr) * gs
            sent = np.isin(sample, idx)
            pos = np.searchsorted(idx, sample[sent])
            assert np.array_equal(bits(val[pos]), bits(p[sent]))
            assert np.array_equal(bits(e_new[sample][~sent]), bits(p[~sent]))
            e_prev[i] = e_new[sample]
            del e_new
        g.aggregate()
        U = g.get_update()[sample]
        acc = np.zeros(len(sample), dtype=F32)
        for i in range(w.n):
            idx, val = g.get_message(i)
            hit = np.isin(sample, idx)
            acc[hit] = acc[hit] + val[np.searchsorted(idx, sample[hit])]
        assert np.array_equal(bits(U), bits(acc))
        x_before = g.get_model()[sample]
        g.apply_delayed(w.lr)
        assert np.array_equal(bits(g.get_model()[sample]), bits(x_before - acc / F32(w.n)))
    # both searches ran at this size: the whole-row one in the first real iteration only
    assert g.full_select_count() == w.n
    g.close()
    c4_problem.cache_clear()


def test_the_longest_vector_the_library_takes(ddef, oracle_mod):
    """One worker with d = 2^32 - 8193, the largest length ddef_init accepts: indices up to 2^32 - 8194
    (far above 2^31), an odd length with a ragged last quad, group, chunk and tile.  Properties of
    the selection plus gradients / error-feedback values on sampled coordinates (the oracle's noise
    is evaluated one coordinate at a time).  The problem vectors are a random block of 2^26 entries
    laid end to end at shifting offsets (the noise differs in every coordinate)."""
    d, n, delta, lr, seed = 2 ** 32 - 8193, 1, 1e-4, 0.05, 77
    with pytest.raises(ddef.DdefError):
        ddef.Context(d + 1, n, 0)                       # one more is rejected before anything is allocated
    rng = np.random.default_rng(5)
    block = 1 << 26
    base = ((10.0 ** rng.uniform(-3, 0, block)).astype(F32), rng.standard_normal(block, dtype=F32),
            rng.standard_normal(block, dtype=F32))
    lam = np.empty(d, dtype=F32); xstar = np.empty(d, dtype=F32); x0 = np.empty(d, dtype=F32)
    for piece, lo in enumerate(range(0, d, block)):
        hi = min(d, lo + block)
        shift = (piece * 1_000_003) % block
        for out, src in zip((lam, xstar, x0), base):
            first = min(hi - lo, block - shift)
            out[lo:lo + first] = src[shift:shift + first]
            out[lo + first:hi] = src[:hi - lo - first]
    c = ddef.Context(d, n, 0)
    c.set_problem(lam, xstar, x0, seed, 1, 0.05)
    c.set_tau(0)
    k = ddef.k_from_delta(delta, d)
    sample = np.unique(np.concatenate([rng.integers(0, d, 3000), rng.integers(d - 10000, d, 50),
                                       [0, d - 1, d - 2, d - 3, d - 4, d - 257, d - 4097, 2 ** 31 - 1, 2 ** 31, 2 ** 31 + 1]]))
    e_prev = np.zeros(len(sample), dtype=F32)
    x_cur = x0
    for t in range(5):
        c.grad()
        c.ef_compress(delta, lr)
        idx, val = c.get_message(0)
        T, r = c.get_threshold(0)
        assert len(idx) == k and np.all(np.diff(idx.astype(np.int64)) > 0) and int(idx[-1]) < d
        assert int((idx >= 2 ** 31).sum()) > k // 4
        vkeys = bits(val) & np.uint32(0x7FFFFFFF)
        assert int(vkeys.min()) == T and int((vkeys == T).sum()) == r
        e_new = c.get_error(0)
        assert int((bits(e_new) & np.uint32(0x7FFFFFFF)).max()) <= T and np.all(bits(e_new[idx]) == 0)
        gs = c.get_grad(0)[sample]
        z = np.array([oracle_mod.noise_z(seed, t, 0, int(j), 1) for j in sample], dtype=F32)
        assert np.array_equal(bits(gs), bits(lam[sample] * (x_cur[sample] - xstar[sample]) + F32(0.05) * z))
        p = e_prev + F32(lr) * gs
        sent = np.isin(sample, idx)
        assert np.array_equal(bits(val[np.searchsorted(idx, sample[sent])]), bits(p[sent]))
        assert np.array_equal(bits(e_new[sample][~sent]), bits(p[~sent]))
        e_prev = e_new[sample]
        del e_new
        c.aggregate()
        c.apply_delayed(lr)
        x_cur = c.get_model()
    assert c.full_select_count() < 5          # the candidate filter carried the later selections
    # one iteration of Random-k at this length (k = 4.3e6 kept coordinates, sorted into regions of
    # 2^21 coordinates before their bits are set): the oracle's subset, the accumulated values there
    del x_cur
    c.set_compressor(1)
    k_r = ddef.k_from_delta(1e-3, d)
    e_before = c.get_error(0)
    c.grad()
    grad = c.get_grad(0)
    c.ef_compress(1e-3, lr)
    idx, val = c.get_message(0)
    assert np.array_equal(idx, oracle_mod.randk_indices(seed, 5, 0, d, k_r))
    some = np.concatenate([np.arange(0, k_r, 997), [k_r - 1]])
    assert np.array_equal(bits(val[some]), bits(e_before[idx[some]] + F32(lr) * grad[idx[some]]))
    p = e_before[sample] + F32(lr) * grad[sample]
    del e_before, grad
    e_new = c.get_error(0)
    unsent = ~np.isin(sample, idx)
    assert np.all(bits(e_new[idx]) == 0) and np.array_equal(bits(e_new[sample][unsent]), bits(p[unsent]))
    del e_new
    c.aggregate()
    c.apply_delayed(lr)
    c.close()


def test_random_k_marking_beyond_2_to_29(ddef, oracle_mod):
    """d = 6e8: the kept coordinates of Random-k are sorted into regions of more than one on-chip
    tile each before their bits are set.  The coordinates sent must be the oracle's subset, the
    values what was accumulated there; the composed compressor on top must send an ordered part
    of that subset."""
    d, n, lr = 600_000_000, 1, 0.05
    w = workloads.replace(workloads.get("C1", d=d, n=n), seed=77)
    lam, xstar, x0 = workloads.make_problem(w)
    c = ddef.Context(d, n, 1)
    c.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    c.set_tau(0)
    k1 = oracle_mod.k_from_delta(0.2, d)
    for comp, delta in ((1, 0.2), (2, 0.1)):
        c.set_compressor(comp)
        c.set_composed(0.2)
        t = c.t
        e_before = c.get_error(0)
        c.grad()
        grad = c.get_grad(0)
        c.ef_compress(delta, lr)
        idx, val = c.get_message(0)
        kept = oracle_mod.randk_indices(w.seed, t, 0, d, k1)
        if comp == 1:
            assert np.array_equal(idx, kept)
            assert np.array_equal(bits(val), bits(e_before[idx] + F32(lr) * grad[idx]))
            assert np.all(bits(c.get_error(0)[idx]) == 0)
        else:
            assert len(idx) == oracle_mod.k_from_delta(delta, k1)
            assert np.all(np.diff(idx.astype(np.int64)) > 0)
            assert np.array_equal(kept[np.searchsorted(kept, idx)], idx)
            p = e_before + F32(lr) * grad
            T, r = c.get_threshold(0)
            keys = bits(p[idx]) & np.uint32(0x7FFFFFFF)
            assert int(keys.min()) == T and int((keys == T).sum()) == r
            unsent = np.setdiff1d(kept, idx, assume_unique=True)
            assert int((bits(p[unsent]) & np.uint32(0x7FFFFFFF)).max()) <= T
        del e_before, grad
        c.aggregate()
        c.apply_delayed(lr)
    assert c.full_select_count() == 0
    c.close()
