"""Pins for the oracle's composed compressor: Random-k, Top-k inside the kept coordinates, 4-bit
codes (Section 5.2 "Baselines": the compressor of the strongest static baseline, given there as the
three stages with their ratios, 20 % and 10 %, and the code width, 4 bits).  The paper says nothing
more about it; the block rule of the quantiser is a reading, pinned here by a hand-worked block, by brute
force over all 15 levels, and by the case where quantisation loses nothing."""
import os

import numpy as np
import pytest

from paper_2507_17346_amd import workloads

F32 = np.float32
HERE = os.path.dirname(os.path.abspath(__file__))


def bits(a):
    return np.asarray(a, dtype=F32).view(np.uint32)


def unpack(codes, k):
    """Signed codes from the packed bytes: low nibble = even position, two's complement."""
    nib = np.empty(2 * len(codes), dtype=np.int64)
    nib[0::2] = codes & 0xF
    nib[1::2] = codes >> 4
    nib = nib[:k]
    return np.where(nib >= 8, nib - 16, nib)


def test_worked_block_from_the_fixture(oracle_mod):
    rows, packed = [], None
    for line in open(os.path.join(HERE, "golden", "quantize4_worked_block.txt")):
        if line.startswith("#"):
            tok = line[1:].split()
            if tok and all(len(t) == 2 and set(t) <= set("0123456789abcdef") for t in tok):
                packed = [int(t, 16) for t in tok]
            continue
        if line.strip():
            v, q, dq = line.split()
            rows.append((float(v), int(q), float(dq)))
    vals = np.array([r[0] for r in rows], dtype=F32)
    codes, steps, deq = oracle_mod.quantize4(vals)
    assert steps.tolist() == [1.0]
    assert unpack(codes, len(rows)).tolist() == [r[1] for r in rows]
    assert deq.tolist() == [r[2] for r in rows]
    assert codes.tolist() == packed
    # -0.5 goes to code 0 and decodes to +0, not -0
    assert bits(deq)[5] == 0


@pytest.mark.parametrize("count", [1, 2, 255, 256, 257, 1000, 5001])
@pytest.mark.parametrize("dist", ["normal", "student_t3", "tiny"])
def test_every_code_is_a_nearest_level(oracle_mod, count, dist):
    rng = np.random.default_rng(count * 7 + len(dist))
    if dist == "normal":
        vals = rng.standard_normal(count)
    elif dist == "student_t3":
        vals = rng.standard_t(3, count)
    else:
        vals = rng.standard_normal(count) * 1e-41          # denormal range: the step is coarse
    vals = vals.astype(F32)
    codes, steps, deq = oracle_mod.quantize4(vals)
    q = unpack(codes, count)
    assert len(codes) == (count + 1) // 2 and len(steps) == (count + 255) // 256
    assert q.min() >= -7 and q.max() <= 7
    levels = np.arange(-7, 8, dtype=np.float64)
    for b in range(len(steps)):
        sl = slice(256 * b, min(count, 256 * b + 256))
        v = vals[sl].astype(np.float64)
        step = float(steps[b])
        largest = np.abs(v).max()
        # the step is the block's largest magnitude over 7, rounded once
        assert step == float(F32(largest) / F32(7.0))
        if step == 0.0:
            assert np.all(q[sl] == 0) and np.all(bits(deq[sl]) == 0)
            continue
        # brute force: no other level is closer (up to the rounding of value / step)
        dist_all = np.abs(v[:, None] - levels[None, :] * step)
        chosen = np.abs(v - q[sl] * step)
        assert np.all(chosen <= dist_all.min(axis=1) + step * 2.0 ** -20)
        # so the error is at most half a step, and the largest entry keeps (nearly) its value
        assert np.all(chosen <= 0.5 * step * (1 + 2.0 ** -20))
        top = np.argmax(np.abs(v))
        assert abs(q[sl][top]) == 7
        # decoded value = code * step in fp32
        assert np.array_equal(bits(deq[sl]), bits(q[sl].astype(F32) * F32(step)))
        # a decoded value never has the other sign, and never a larger magnitude than 7 steps
        assert np.all(deq[sl].astype(np.float64) * v >= 0)


def test_halves_go_to_the_even_code(oracle_mod):
    vals = np.array([7, 0.5, 1.5, 2.5, 3.5, 4.5, 5.5, 6.5, -0.5, -1.5, -2.5, -3.5, -4.5, -5.5, -6.5], dtype=F32)
    codes, steps, deq = oracle_mod.quantize4(vals)
    assert unpack(codes, len(vals)).tolist() == [7, 0, 2, 2, 4, 4, 6, 6, 0, -2, -2, -4, -4, -6, -6]


def test_blocks_have_their_own_step(oracle_mod):
    vals = np.concatenate([np.full(256, 14.0), np.full(256, 0.0), np.full(10, -3.5)]).astype(F32)
    vals[300] = 0.0
    codes, steps, deq = oracle_mod.quantize4(vals)
    assert steps.tolist() == [2.0, 0.0, 0.5]
    q = unpack(codes, len(vals))
    assert np.all(q[:256] == 7) and np.all(q[256:512] == 0) and np.all(q[512:] == -7)
    assert np.array_equal(deq, vals)


def make(oracle_mod, d, n, tau, seed, rand_ratio, noise_kind=1, noise_scale=0.1):
    w = workloads.replace(workloads.get("C1", d=d, n=n), seed=seed, noise_kind=noise_kind, noise_scale=noise_scale)
    lam, xstar, x0 = workloads.make_problem(w)
    o = oracle_mod.Oracle(d, n, tau)
    o.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    o.set_tau(tau)
    o.set_compressor(2)
    o.set_composed(rand_ratio)
    return o, w, x0


def test_selection_is_the_top_of_the_random_subset(oracle_mod):
    # indices against a numpy sort of the kept coordinates; values, residual and update against
    # what the three stages mean; conservation over the run
    d, n, tau, lr, rho, delta = 5000, 3, 1, 0.05, 0.2, 0.1
    o, w, x0 = make(oracle_mod, d, n, tau, 31, rho)
    k1 = oracle_mod.k_from_delta(rho, d)
    k = oracle_mod.k_from_delta(delta, k1)
    assert (k1, k) == (1000, 100)
    sent = np.zeros((n, d))
    fed = np.zeros((n, d))
    x = x0.copy()
    for t in range(12):
        e_before = [o.get_error(i) for i in range(n)]
        o.grad()
        o.ef_compress(delta, lr)
        U = np.zeros(d, dtype=F32)
        for i in range(n):
            idx, val = o.get_message(i)
            if t < tau:
                assert len(idx) == 0
                continue
            p = e_before[i] + F32(lr) * o.get_grad(i)
            subset = oracle_mod.randk_indices(w.seed, t, i, d, k1)
            key = bits(p[subset]) & 0x7FFFFFFF
            order = np.lexsort((subset, -key.astype(np.int64)))      # magnitude descending, coordinate ascending
            want = np.sort(subset[order[:k]])
            assert np.array_equal(idx, want)
            T, r = o.get_threshold(i)
            assert T == int(key[order[k - 1]]) and r == int((key[order[:k]] == T).sum())
            codes, steps = o.get_message_codes(i)
            c2, s2, deq = oracle_mod.quantize4(p[idx])
            assert np.array_equal(codes, c2) and np.array_equal(bits(steps), bits(s2))
            assert np.array_equal(bits(val), bits(deq))
            e_after = o.get_error(i)
            mask = np.ones(d, dtype=bool)
            mask[idx] = False
            assert np.array_equal(bits(e_after[mask]), bits(p[mask]))
            # sent + kept error gives p back (one rounding of the subtraction)
            assert np.all(np.abs(val.astype(np.float64) + e_after[idx] - p[idx]) <= 2.0 ** -23 * np.abs(p[idx]))
            # contraction: what is kept back is never larger than what came in
            assert np.all(np.abs(e_after) <= np.abs(p))
            sent[i, idx] += val.astype(np.float64)
            fed[i] += float(F32(lr)) * o.get_grad(i).astype(np.float64)
            U[idx] = U[idx] + val
        o.aggregate()
        assert np.array_equal(bits(o.get_update()), bits(U))
        o.apply_delayed()
        x = x - U / F32(n)
        assert np.array_equal(bits(o.get_model()), bits(x))
    for i in range(n):
        assert np.abs(sent[i] + o.get_error(i) - fed[i]).max() <= 20 * 2.0 ** -22 * np.abs(fed).max()


def test_values_on_the_grid_make_it_plain_top_k(oracle_mod):
    # rand_ratio = 1 keeps every coordinate; gradients that are integers in [-7, 7] times a power of
    # two, with a +-7 in every block of the message, lose nothing in the 4-bit stage: message,
    # residual and model must equal the Top-k compressor's (pinned on its own elsewhere)
    d, n, k = 4096, 2, 1024
    rng = np.random.default_rng(5)
    results = []
    for kind in (2, 0):
        w = workloads.replace(workloads.get("C1", d=d, n=n), seed=3, noise_kind=0, noise_scale=0.0)
        lam, xstar, x0 = workloads.make_problem(w)
        o = oracle_mod.Oracle(d, n, 0)
        o.set_problem(lam, xstar, x0, w.seed, 0, 0.0)
        o.set_tau(0)
        o.set_compressor(kind)
        o.set_composed(1.0)
        rng = np.random.default_rng(5)
        for i in range(n):
            g = rng.integers(-3, 4, d).astype(F32)            # the crowd: |g| <= 3
            big = rng.choice(d, k, replace=False)
            g[big] = rng.choice([-7, -6, -5, -4, 4, 5, 6, 7], k).astype(F32)
            g[np.sort(big)[::64]] = 7.0                        # a 7 in every 64 message entries
            o.load_grad(i, g * F32(0.25))
        o.ef_compress(k / d, 1.0)
        o.aggregate()
        o.apply_delayed()
        results.append(([o.get_message(i) for i in range(n)], [o.get_error(i) for i in range(n)], o.get_model()))
    (m2, e2, x2), (m0, e0, x0_) = results
    for i in range(n):
        assert np.array_equal(m2[i][0], m0[i][0])
        assert np.array_equal(bits(m2[i][1]), bits(m0[i][1]))
        assert np.array_equal(bits(e2[i]), bits(e0[i]))
    assert np.array_equal(bits(x2), bits(x0_))


def test_sizes_follow_the_two_ratios(oracle_mod):
    for d, rho, delta in [(10, 0.2, 0.1), (3, 0.2, 0.1), (1000, 0.2, 0.1), (1000, 1.0, 1.0), (999, 0.333, 0.5)]:
        o, w, x0 = make(oracle_mod, d, 2, 0, 7, rho)
        o.grad()
        o.ef_compress(delta, 0.05)
        k1 = oracle_mod.k_from_delta(rho, d)
        k = oracle_mod.k_from_delta(delta, k1)
        idx, val = o.get_message(0)
        assert len(idx) == k and len(np.unique(idx)) == k
        assert set(idx.tolist()) <= set(oracle_mod.randk_indices(w.seed, 0, 0, d, k1).tolist())
