"""Pins for the oracle's DD-EF-SGD step against what the paper and the mathematics fix:
degenerate cases (Section 2.2), the error-feedback bookkeeping of Algorithm 1, the nested
virtual sequence identity (Section 3.2), the Top-k contraction, the closed form on the
noiseless quadratic, and the equivalence of the snapshot-ring form with Algorithm 1 as
printed (message queue)."""
import numpy as np
import pytest

from paper_2507_17346_amd import workloads

F32 = np.float32


def small_problem(seed=0, d=3000, n=3, noise_kind=1, noise_scale=0.1):
    w = workloads.get("C1", d=d, n=n)
    w = workloads.replace(w, seed=seed, noise_kind=noise_kind, noise_scale=noise_scale)
    lam, xstar, x0 = workloads.make_problem(w)
    return w, lam, xstar, x0


def make_oracle(oracle_mod, w, lam, xstar, x0, tau, tau_max=None):
    o = oracle_mod.Oracle(w.d, w.n, tau if tau_max is None else tau_max)
    o.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    o.set_tau(tau)
    return o


def bits(a):
    return np.asarray(a, dtype=F32).view(np.uint32)


# --- P2 / P5: per-step EF identity, bit exact, and the contraction bound -------------------
@pytest.mark.parametrize("delta,tau", [(0.01, 0), (0.05, 2), (0.3, 1), (1.0, 0)])
def test_ef_identity_and_contraction_every_step(oracle_mod, delta, tau):
    w, lam, xstar, x0 = small_problem(seed=3)
    o = make_oracle(oracle_mod, w, lam, xstar, x0, tau)
    lr = 0.05
    k = oracle_mod.k_from_delta(delta, w.d)
    for t in range(8):
        e_before = [o.get_error(i) for i in range(w.n)]
        o.grad()
        o.ef_compress(delta, lr)
        for i in range(w.n):
            idx, val = o.get_message(i)
            e_after = o.get_error(i)
            if t < tau:
                assert len(idx) == 0 and np.array_equal(bits(e_after), bits(e_before[i]))
                continue
            g = o.get_grad(i)
            p = e_before[i] + F32(lr) * g                      # numpy fp32: two roundings
            assert len(idx) == k and np.all(np.diff(idx.astype(np.int64)) > 0)
            dense = np.zeros(w.d, dtype=F32)
            dense[idx] = val
            assert np.array_equal(bits(val), bits(p[idx]))
            # supports are disjoint and Delta + e' == p as bit patterns (+0 where selected)
            assert np.all(bits(e_after[idx]) == 0)
            mask = np.ones(w.d, dtype=bool)
            mask[idx] = False
            assert np.array_equal(bits(e_after[mask]), bits(p[mask]))
            p64 = p.astype(np.float64)
            assert (e_after.astype(np.float64) ** 2).sum() <= (1 - k / w.d) * (p64 ** 2).sum() * (1 + 1e-12)
        o.aggregate()
        o.apply_delayed()


# --- P3 / P4: conservation and the virtual-sequence identity -------------------------------
@pytest.mark.parametrize("tau", [0, 3])
def test_conservation_and_virtual_sequence(oracle_mod, tau):
    w, lam, xstar, x0 = small_problem(seed=4, d=2000, n=4)
    o = make_oracle(oracle_mod, w, lam, xstar, x0, tau)
    lr, delta, steps = 0.05, 0.02, 30
    sent = np.zeros((w.n, w.d))
    fed = np.zeros((w.n, w.d))
    for t in range(steps):
        o.grad()
        o.ef_compress(delta, lr)
        for i in range(w.n):
            idx, val = o.get_message(i)
            sent[i, idx] += val.astype(np.float64)
            if t >= tau:
                fed[i] += float(F32(lr)) * o.get_grad(i).astype(np.float64)
        o.aggregate()
        o.apply_delayed()
    scale = np.abs(fed).max()
    for i in range(w.n):
        # sum of everything sent + what is still held back = sum of lr * g fed in
        assert np.abs(sent[i] + o.get_error(i) - fed[i]).max() <= steps * 2.0 ** -22 * scale
    # x_T - (1/n) sum_i e_i = x_0 - (1/n) sum_i sum lr*g   (the error buffers hold what the
    # model has not yet received; no stepsize factor on the error term)
    x_hat = o.get_model().astype(np.float64) - sum(o.get_error(i).astype(np.float64) for i in range(w.n)) / w.n
    want = x0.astype(np.float64) - fed.sum(axis=0) / w.n
    assert np.abs(x_hat - want).max() <= steps * 2.0 ** -21 * max(scale, np.abs(x0).max())


# --- P7: delta = 1, tau = 0 is D-SGD ---------------------------------------------------------
def test_delta_one_tau_zero_is_dsgd(oracle_mod):
    w, lam, xstar, x0 = small_problem(seed=5, d=1500, n=4)
    o = make_oracle(oracle_mod, w, lam, xstar, x0, 0)
    lr = 0.05
    x = x0.copy()
    x_text = x0.astype(np.float64)
    for t in range(12):
        o.grad()
        gs = [o.get_grad(i) for i in range(w.n)]
        # the gradient itself: lambda * (x - x*) + scale * z, rounded after every operation
        for i in range(w.n):
            z = oracle_mod.noise_fill(w.seed, t, i, 0, w.d, w.noise_kind)
            assert np.array_equal(bits(gs[i]), bits(lam * (x - xstar) + F32(w.noise_scale) * z))
        o.ef_compress(1.0, lr)
        o.aggregate()
        o.apply_delayed()
        acc = np.zeros(w.d, dtype=F32)
        for i in range(w.n):
            acc = acc + F32(lr) * gs[i]
            assert np.all(bits(o.get_error(i)) == 0)           # nothing is ever held back
        x = x - acc / F32(w.n)
        assert np.array_equal(bits(o.get_model()), bits(x))
        # textbook D-SGD x - (lr/n) sum g, in double
        x_text = x_text - (lr / w.n) * sum(g.astype(np.float64) for g in gs)
    assert np.abs(o.get_model() - x_text).max() <= 1e-6 * np.abs(x_text).max()


# --- P8: delta = 1, tau > 0 is delayed-aggregation SGD ---------------------------------------
def test_delta_one_is_delayed_sgd(oracle_mod):
    tau = 3
    w, lam, xstar, x0 = small_problem(seed=6, d=1200, n=2)
    o = make_oracle(oracle_mod, w, lam, xstar, x0, tau)
    lr = 0.05
    hist = [x0.astype(np.float64)]
    for t in range(15):
        o.grad()
        o.ef_compress(1.0, lr)
        o.aggregate()
        o.apply_delayed()
        if t < tau:
            nxt = hist[-1].copy()
        else:
            xs = hist[t - tau].astype(F32)
            g = [(lam * (xs - xstar) + F32(w.noise_scale) * oracle_mod.noise_fill(w.seed, t, i, 0, w.d, 1)).astype(np.float64)
                 for i in range(w.n)]
            nxt = hist[-1] - (lr / w.n) * sum(g)
        hist.append(nxt.astype(F32).astype(np.float64))
        assert np.abs(o.get_model() - hist[-1]).max() <= 1e-6 * np.abs(hist[-1]).max()


# --- P8: tau = 0, delta < 1: the three update rules of Section 2.2.2 --------------------------
def test_tau_zero_is_ef_compressed_sgd(oracle_mod):
    w, lam, xstar, x0 = small_problem(seed=7, d=800, n=3)
    o = make_oracle(oracle_mod, w, lam, xstar, x0, 0)
    lr, delta = 0.05, 0.05
    k = oracle_mod.k_from_delta(delta, w.d)
    x = x0.copy()
    e = [np.zeros(w.d, dtype=F32) for _ in range(w.n)]
    for t in range(10):
        upd = np.zeros(w.d, dtype=F32)
        for i in range(w.n):
            g = lam * (x - xstar) + F32(w.noise_scale) * oracle_mod.noise_fill(w.seed, t, i, 0, w.d, 1)
            p = e[i] + F32(lr) * g
            keys = bits(p) & np.uint32(0x7FFFFFFF)
            order = np.lexsort((np.arange(w.d), -keys.astype(np.int64)))   # stable: |v| desc, index asc
            comp = np.zeros(w.d, dtype=F32)
            comp[order[:k]] = p[order[:k]]
            e[i] = p - comp
            upd = upd + comp
        x = x - upd / F32(w.n)
        o.step(delta, lr)
        assert np.array_equal(bits(o.get_model()), bits(x))
        for i in range(w.n):
            assert np.array_equal(bits(o.get_error(i)), bits(e[i]))


# --- P9: closed form on the noiseless quadratic ---------------------------------------------
def test_closed_form_noiseless(oracle_mod):
    w, lam, xstar, x0 = small_problem(seed=8, d=500, n=2, noise_kind=0, noise_scale=0.0)
    lr, steps = 0.05, 40
    o = make_oracle(oracle_mod, w, lam, xstar, x0, 0)
    for _ in range(steps):
        o.step(1.0, lr)
    z0 = x0.astype(np.float64) - xstar
    want = xstar + (1.0 - lr * lam.astype(np.float64)) ** steps * z0
    assert np.abs(o.get_model() - want).max() <= steps * 2.0 ** -22 * np.abs(want).max()
    # with delay: z_{t+1} = z_t - lr*lambda*z_{t-tau}, z_t = z_0 for t <= tau
    tau = 4
    o = make_oracle(oracle_mod, w, lam, xstar, x0, tau)
    for _ in range(steps):
        o.step(1.0, lr)
    z = [z0.copy()]
    for t in range(steps):
        z.append(z[-1] if t < tau else z[-1] - lr * lam.astype(np.float64) * z[t - tau])
    want = xstar + z[-1]
    assert np.abs(o.get_model() - want).max() <= steps * 2.0 ** -22 * np.abs(want).max()


# --- P6: snapshot ring == Algorithm 1 as printed (message queue), constant tau ---------------
@pytest.mark.parametrize("tau,delta", [(0, 0.1), (1, 0.02), (3, 0.05), (5, 1.0)])
def test_ring_form_equals_queue_form(oracle_mod, tau, delta):
    w, lam, xstar, x0 = small_problem(seed=9 + tau, d=700, n=3)
    lr, T = 0.05, 14
    o = make_oracle(oracle_mod, w, lam, xstar, x0, tau)
    _, traj = oracle_mod.queue_run(lam, xstar, x0, w.n, tau, T, delta, lr, w.seed, w.noise_kind,
                                   w.noise_scale, trajectory=True)
    assert np.array_equal(bits(traj[0]), bits(x0))
    for t in range(T):
        o.step(delta, lr)
        assert np.array_equal(bits(o.get_model()), bits(traj[t + 1])), t
    for t in range(tau + 1):                       # nothing arrives before step tau
        assert np.array_equal(bits(traj[t]), bits(x0))
    assert not np.array_equal(bits(traj[tau + 1]), bits(x0))


# --- start-up and a changing tau (Algorithm 2): invariants only -----------------------------
def test_startup_noop_steps_and_snapshot_ring(oracle_mod):
    tau = 2
    w, lam, xstar, x0 = small_problem(seed=12, d=300, n=2)
    o = make_oracle(oracle_mod, w, lam, xstar, x0, tau, tau_max=4)
    for t in range(tau):
        o.step(0.1, 0.05)
        assert o.t == t + 1
        assert np.array_equal(bits(o.get_model()), bits(x0))
        assert np.all(bits(o.get_update()) == 0)
    o.step(0.1, 0.05)
    assert not np.array_equal(bits(o.get_model()), bits(x0))
    # grow tau: the gradient of step t is taken at the snapshot x_{t - tau}
    snaps = {s: o.get_snapshot(s) for s in range(0, o.t + 1)}
    o.set_tau(3)
    o.grad()
    xs = snaps[o.t - 3]
    z = oracle_mod.noise_fill(w.seed, o.t, 1, 0, w.d, 1)
    assert np.array_equal(bits(o.get_grad(1)), bits(lam * (xs - xstar) + F32(w.noise_scale) * z))


def test_gradient_does_not_depend_on_the_number_of_threads(oracle_mod):
    """With more threads than workers the oracle's threads share each worker's coordinates in
    ranges.  Every coordinate must still be computed, and computed as lambda (x - x*) + scale z
    (Assumption 2) from the noise draws taken one by one."""
    w, lam, xstar, x0 = small_problem(seed=21, d=1003, n=2, noise_kind=2, noise_scale=0.3)
    want = None
    for threads in (1, 2, 5, 7, 16):
        o = oracle_mod.Oracle(w.d, w.n, 0, threads=threads)
        o.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
        o.set_tau(0)
        for i in range(w.n):
            o.set_error(i, np.full(w.d, np.nan, dtype=F32))      # (the gradient does not read it)
        o.grad()
        got = [o.get_grad(i) for i in range(w.n)]
        if want is None:
            want = got
            for i in range(w.n):
                z = oracle_mod.noise_fill(w.seed, 0, i, 0, w.d, w.noise_kind)
                assert np.array_equal(bits(got[i]), bits(lam * (x0 - xstar) + F32(w.noise_scale) * z))
        for i in range(w.n):
            assert np.array_equal(bits(got[i]), bits(want[i])), (threads, i)
        o.close()


def test_a_new_problem_starts_from_empty_error_buffers(oracle_mod):
    """e_0 = 0 (Algorithm 1's initialisation): handing the problem over again restarts the run."""
    w, lam, xstar, x0 = small_problem(seed=22, d=700, n=2)
    o = make_oracle(oracle_mod, w, lam, xstar, x0, 1)
    first = []
    for _ in range(4):
        o.step(0.05, 0.05)
        first.append(o.get_model())
    assert any(np.any(o.get_error(i) != 0) for i in range(w.n))
    o.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    assert o.t == 0 and all(not np.any(o.get_error(i)) for i in range(w.n))
    for t in range(4):
        o.step(0.05, 0.05)
        assert np.array_equal(bits(o.get_model()), bits(first[t])), t
    o.close()


def test_aggregate_sums_in_worker_order(oracle_mod):
    # three workers whose selected values do not add associatively in fp32
    d, n = 4, 3
    o = oracle_mod.Oracle(d, n, 0)
    zero = np.zeros(d, dtype=F32)
    o.set_problem(np.ones(d, dtype=F32), zero, zero, 0, 0, 0.0)
    vals = [F32(1e8), F32(-1e8), F32(1.0)]
    for i in range(n):
        g = np.zeros(d, dtype=F32)
        g[2] = vals[i]
        g[i % 2] = F32(0.5)
        o.load_grad(i, g)
    o.ef_compress(0.5, 1.0)
    o.aggregate()
    U = o.get_update()
    assert U[2] == (F32(1e8) + F32(-1e8)) + F32(1.0) == F32(1.0)
    assert U[0] == F32(1.0) and U[1] == F32(0.5) and U[3] == 0.0
    o.apply_delayed()
    assert np.array_equal(o.get_model(), -U / F32(3))


# --- the literal form one iteration at a time: same x as the batch run and as the ring form ---------
@pytest.mark.parametrize("tau,delta", [(0, 0.05), (2, 0.03), (4, 0.2)])
def test_stepwise_queue_form(oracle_mod, tau, delta):
    w, lam, xstar, x0 = small_problem(seed=40 + tau, d=900, n=3)
    lr, T = 0.05, 12
    q = oracle_mod.QueueOracle(w.d, w.n, tau)
    q.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    ring = make_oracle(oracle_mod, w, lam, xstar, x0, tau)
    _, traj = oracle_mod.queue_run(lam, xstar, x0, w.n, tau, T, delta, lr, w.seed, w.noise_kind,
                                   w.noise_scale, trajectory=True)
    for t in range(T):
        q.step(delta, lr)
        ring.step(delta, lr)
        assert np.array_equal(bits(q.get_model()), bits(traj[t + 1]))
        assert np.array_equal(bits(q.get_model()), bits(ring.get_model()))
    # the message the queue form sends at time t is the one the ring form computes at t + tau, and
    # the queue form's error buffers run tau iterations ahead of the ring form's
    q2 = oracle_mod.QueueOracle(w.d, w.n, tau)
    q2.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    ring2 = make_oracle(oracle_mod, w, lam, xstar, x0, tau)
    for t in range(tau):
        ring2.step(delta, lr)                      # the ring form's empty start-up iterations
    for t in range(T - tau):
        q2.step(delta, lr)
        ring2.step(delta, lr)
        for i in range(w.n):
            qi, qv = q2.get_message(i)
            ri, rv = ring2.get_message(i)
            assert np.array_equal(qi, ri) and np.array_equal(bits(qv), bits(rv))
            assert np.array_equal(bits(q2.get_error(i)), bits(ring2.get_error(i)))


def queue_noise_keys(taus):
    """Noise key of the gradient taken at iteration u in the message-queue form: the iteration
    u + tau_u at which its message is due, pushed up so that the keys never repeat."""
    keys, floor = [], 0
    for u, tau in enumerate(taus):
        keys.append(max(u + tau, floor))
        floor = keys[-1] + 1
    return keys


def topk_dense(p, k):
    """Top-k of p as a dense vector, by a full stable sort: |v| descending on the bit pattern with
    the sign cleared, lower index first among equals."""
    keys = bits(p) & np.uint32(0x7FFFFFFF)
    order = np.lexsort((np.arange(len(p)), -keys.astype(np.int64)))
    comp = np.zeros(len(p), dtype=F32)
    comp[order[:k]] = p[order[:k]]
    return comp, np.sort(order[:k]).astype(np.uint32)


# (tau_t, delta_t) re-chosen as Algorithm 2 does every E iterations, here every 3: tau rises, falls
# and returns, delta changes with it
CHANGING = [(2, 0.05)] * 3 + [(0, 0.2)] * 3 + [(4, 0.02)] * 3 + [(1, 0.1)] * 3 + [(3, 0.05)] * 3 + \
           [(3, 0.3)] * 2 + [(0, 0.01)] * 2 + [(4, 0.2)] * 3


def test_ring_form_changing_tau_and_delta_numpy_replay(oracle_mod):
    """Algorithm 2 re-chooses (tau, delta) while Algorithm 1 runs.  In the snapshot-ring form
    iteration t takes every worker's gradient at x_{t - tau_t} with the noise of iteration t, runs
    error feedback and Top-k with k_t = ceil(delta_t d), and applies the sum at once; while
    t - tau_t < 0 nothing arrives (Section 3.2's convention): x and every e_i stay.  Replayed here
    in numpy from a list of all iterates; messages, error buffers, update and model bit for bit."""
    w, lam, xstar, x0 = small_problem(seed=71, d=900, n=3)
    lr = 0.05
    o = make_oracle(oracle_mod, w, lam, xstar, x0, 0, tau_max=4)
    xs = [x0.copy()]
    e = [np.zeros(w.d, dtype=F32) for _ in range(w.n)]
    real = 0
    for t, (tau, delta) in enumerate(CHANGING):
        k = int(np.ceil(delta * w.d))
        o.set_tau(tau)
        o.step(delta, lr)
        upd = np.zeros(w.d, dtype=F32)
        if t - tau >= 0:
            real += 1
            stale = xs[t - tau]
            for i in range(w.n):
                z = oracle_mod.noise_fill(w.seed, t, i, 0, w.d, w.noise_kind)
                g = lam * (stale - xstar) + F32(w.noise_scale) * z
                p = e[i] + F32(lr) * g
                comp, chosen = topk_dense(p, k)
                e[i] = p - comp
                upd = upd + comp
                idx, val = o.get_message(i)
                assert np.array_equal(idx, chosen), (t, i)
                assert np.array_equal(bits(val), bits(p[chosen])), (t, i)
        else:
            assert all(len(o.get_message(i)[0]) == 0 for i in range(w.n))
        xs.append(xs[-1] - upd / F32(w.n))
        assert np.array_equal(bits(o.get_update()), bits(upd)), t
        assert np.array_equal(bits(o.get_model()), bits(xs[-1])), t
        for i in range(w.n):
            assert np.array_equal(bits(o.get_error(i)), bits(e[i])), (t, i)
    assert real == len(CHANGING) - 2                               # the first two were empty


def test_stepwise_queue_form_changing_tau_and_delta_numpy_replay(oracle_mod):
    """Algorithm 1 as printed under a changing (tau, delta): every iteration u each worker takes its
    gradient at the current x_u, compresses e + lr*g with k_u = ceil(delta_u d) and sends; the
    server applies what was sent tau_u iterations before u (possibly a message a second time, or
    never), nothing while u - tau_u < 0."""
    w, lam, xstar, x0 = small_problem(seed=72, d=800, n=3)
    lr = 0.05
    taus = [tau for tau, _ in CHANGING]
    keys = queue_noise_keys(taus)
    assert len(set(keys)) == len(keys)
    q = oracle_mod.QueueOracle(w.d, w.n, 0)
    q.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    x = x0.copy()
    e = [np.zeros(w.d, dtype=F32) for _ in range(w.n)]
    sent = []
    for u, (tau, delta) in enumerate(CHANGING):
        k = int(np.ceil(delta * w.d))
        q.set_tau(tau)
        q.step(delta, lr)
        msgs = []
        for i in range(w.n):
            z = oracle_mod.noise_fill(w.seed, keys[u], i, 0, w.d, w.noise_kind)
            g = lam * (x - xstar) + F32(w.noise_scale) * z
            p = e[i] + F32(lr) * g
            comp, chosen = topk_dense(p, k)
            e[i] = p - comp
            msgs.append(comp)
            idx, val = q.get_message(i)
            assert np.array_equal(idx, chosen) and np.array_equal(bits(val), bits(p[chosen])), (u, i)
            assert np.array_equal(bits(q.get_error(i)), bits(e[i])), (u, i)
        sent.append(msgs)
        upd = np.zeros(w.d, dtype=F32)
        if u - tau >= 0:
            for i in range(w.n):
                upd = upd + sent[u - tau][i]
        x = x - upd / F32(w.n)
        assert np.array_equal(bits(q.get_update()), bits(upd)), u
        assert np.array_equal(bits(q.get_model()), bits(x)), u


def test_stepwise_queue_form_changing_tau_is_delayed_sgd_at_delta_one(oracle_mod):
    """delta = 1 keeps every e_i at zero, so the message of iteration u is lr * g_u and the server's
    rule is x_{t+1} = x_t - (1/n) sum_i lr * g_{i, t - tau_t}: replayed here in numpy."""
    w, lam, xstar, x0 = small_problem(seed=61, d=700, n=2)
    lr = 0.05
    taus = [0, 0, 2, 2, 1, 3, 3, 0, 2, 1, 1, 3]
    q = oracle_mod.QueueOracle(w.d, w.n, 0)
    q.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    x = x0.copy()
    sent = []
    keys = queue_noise_keys(taus)
    assert len(set(keys)) == len(keys) and keys[:4] == [0, 1, 4, 5]
    for t, tau in enumerate(taus):
        q.set_tau(tau)
        q.step(1.0, lr)
        msgs = []
        for i in range(w.n):
            z = oracle_mod.noise_fill(w.seed, keys[t], i, 0, w.d, w.noise_kind)
            msgs.append(F32(lr) * (lam * (x - xstar) + F32(w.noise_scale) * z))
            assert np.all(bits(q.get_error(i)) == 0)
            idx, val = q.get_message(i)
            assert np.array_equal(idx, np.arange(w.d)) and np.array_equal(bits(val), bits(msgs[i]))
        sent.append(msgs)
        upd = np.zeros(w.d, dtype=F32)
        if t >= tau:
            for i in range(w.n):
                upd = upd + sent[t - tau][i]
        x = x - upd / F32(w.n)
        assert np.array_equal(bits(q.get_update()), bits(upd))
        assert np.array_equal(bits(q.get_model()), bits(x))


def test_stepwise_queue_form_non_iid_matches_ring_form(oracle_mod):
    tau, delta, lr, T = 2, 0.05, 0.05, 10
    w, lam, xstar, x0 = small_problem(seed=62, d=600, n=3)
    q = oracle_mod.QueueOracle(w.d, w.n, tau)
    q.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    q.set_heterogeneity(0.7)
    ring = make_oracle(oracle_mod, w, lam, xstar, x0, tau)
    ring.set_heterogeneity(0.7)
    for t in range(T):
        q.step(delta, lr)
        ring.step(delta, lr)
        assert np.array_equal(bits(q.get_model()), bits(ring.get_model()))
    plain = oracle_mod.QueueOracle(w.d, w.n, tau)
    plain.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    for t in range(T):
        plain.step(delta, lr)
    assert not np.array_equal(bits(plain.get_model()), bits(q.get_model()))


def test_ring_form_changing_tau_is_delayed_sgd_at_delta_one(oracle_mod):
    """Ring form under a changing tau, delta = 1 (every e_i stays zero): iteration t applies
    lr * g(x_{t - tau_t}) with the noise of iteration t, or nothing while t - tau_t < 0: replayed in
    numpy from the stored iterates."""
    w, lam, xstar, x0 = small_problem(seed=63, d=650, n=3)
    lr = 0.05
    taus = [0, 1, 1, 3, 2, 0, 3, 3, 1, 2, 0, 1]
    o = make_oracle(oracle_mod, w, lam, xstar, x0, 0, tau_max=3)
    xs = [x0.copy()]
    for t, tau in enumerate(taus):
        o.set_tau(tau)
        o.step(1.0, lr)
        x = xs[-1]
        upd = np.zeros(w.d, dtype=F32)
        if t - tau >= 0:
            stale = xs[t - tau]
            for i in range(w.n):
                z = oracle_mod.noise_fill(w.seed, t, i, 0, w.d, w.noise_kind)
                upd = upd + F32(lr) * (lam * (stale - xstar) + F32(w.noise_scale) * z)
        xs.append(x - upd / F32(w.n))
        assert np.array_equal(bits(o.get_update()), bits(upd)), t
        assert np.array_equal(bits(o.get_model()), bits(xs[-1])), t
        for i in range(w.n):
            assert np.all(bits(o.get_error(i)) == 0)
