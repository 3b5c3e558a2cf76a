"""Pins for the oracle's Random-k sparsifier (the paper's appendix on other sparsifiers: "randomly
selects k% gradient elements to transmit"): exactly k distinct coordinates, every coordinate
equally likely, a fresh draw per worker and iteration, and the same error-feedback bookkeeping as
with Top-k."""
import numpy as np
import pytest
from scipy import stats

from paper_2507_17346_amd import workloads

F32 = np.float32


def bits(a):
    return np.asarray(a, dtype=F32).view(np.uint32)


def test_round_function_known_values(oracle_mod):
    # MurmurHash3's 32-bit finaliser: 0 is a fixed point, fmix32(1) = 0x514E28B7 (reference value)
    assert oracle_mod.murmur_fmix32(0) == 0
    assert oracle_mod.murmur_fmix32(1) == 0x514E28B7
    # it is a bijection of 32-bit words: distinct inputs, distinct outputs
    outs = {oracle_mod.murmur_fmix32(x) for x in range(20000)}
    assert len(outs) == 20000


@pytest.mark.parametrize("d", [1, 2, 3, 7, 16, 17, 64, 1000, 4097])
def test_permutation_is_a_bijection(oracle_mod, d):
    for seed, t, worker in [(0, 0, 0), (5, 17, 3), ((1 << 40) + 9, (1 << 33) + 1, 15)]:
        perm = [oracle_mod.randk_permute(seed, t, worker, d, m) for m in range(d)]
        assert sorted(perm) == list(range(d))


def test_indices_are_the_first_k_images_sorted(oracle_mod):
    seed, t, worker, d = 11, 4, 2, 5000
    perm = [oracle_mod.randk_permute(seed, t, worker, d, m) for m in range(d)]
    for k in [1, 2, 50, 4999, 5000]:
        idx = oracle_mod.randk_indices(seed, t, worker, d, k)
        assert idx.tolist() == sorted(perm[:k])
        assert len(np.unique(idx)) == k and int(idx.max()) < d
    assert oracle_mod.randk_indices(seed, t, worker, d, d).tolist() == list(range(d))


def test_every_coordinate_equally_likely(oracle_mod):
    d, k, draws = 200, 20, 3000
    counts = np.zeros(d)
    pair = 0
    for t in range(draws):
        idx = oracle_mod.randk_indices(3, t, 1, d, k)
        counts[idx] += 1
        pair += int(0 in idx and 1 in idx)
    # inclusion probability k/d for every coordinate
    expected = draws * k / d
    chi2 = ((counts - expected) ** 2 / (expected * (1 - k / d))).sum()
    assert stats.chi2.sf(chi2, d - 1) > 1e-3
    # two given coordinates together: k(k-1) / (d(d-1))
    want = draws * k * (k - 1) / (d * (d - 1))
    assert abs(pair - want) < 5 * np.sqrt(want)


def test_draws_differ_between_workers_and_iterations(oracle_mod):
    d, k = 100_000, 1000
    base = set(oracle_mod.randk_indices(1, 5, 0, d, k).tolist())
    for other in (oracle_mod.randk_indices(1, 6, 0, d, k), oracle_mod.randk_indices(1, 5, 1, d, k),
                  oracle_mod.randk_indices(2, 5, 0, d, k)):
        overlap = len(base & set(other.tolist()))
        assert overlap < 40                    # expected k*k/d = 10
    assert base == set(oracle_mod.randk_indices(1, 5, 0, d, k).tolist())


def make(oracle_mod, d, n, tau, seed=0, noise_kind=1, noise_scale=0.1):
    w = workloads.replace(workloads.get("C1", d=d, n=n), seed=seed, noise_kind=noise_kind, noise_scale=noise_scale)
    lam, xstar, x0 = workloads.make_problem(w)
    o = oracle_mod.Oracle(d, n, tau)
    o.set_problem(lam, xstar, x0, w.seed, w.noise_kind, w.noise_scale)
    o.set_tau(tau)
    o.set_compressor(1)
    return o, w, lam, xstar, x0


def test_step_with_random_k_keeps_the_ef_bookkeeping(oracle_mod):
    o, w, lam, xstar, x0 = make(oracle_mod, 3000, 3, 1, seed=21)
    lr, delta = 0.05, 0.04
    k = oracle_mod.k_from_delta(delta, w.d)
    sent = np.zeros((w.n, w.d))
    fed = np.zeros((w.n, w.d))
    for t in range(10):
        e_before = [o.get_error(i) for i in range(w.n)]
        o.grad()
        o.ef_compress(delta, lr)
        for i in range(w.n):
            idx, val = o.get_message(i)
            if t < 1:
                assert len(idx) == 0
                continue
            assert np.array_equal(idx, oracle_mod.randk_indices(w.seed, t, i, w.d, k))
            p = e_before[i] + F32(lr) * o.get_grad(i)
            assert np.array_equal(bits(val), bits(p[idx]))
            e_after = o.get_error(i)
            assert np.all(bits(e_after[idx]) == 0)
            mask = np.ones(w.d, dtype=bool)
            mask[idx] = False
            assert np.array_equal(bits(e_after[mask]), bits(p[mask]))
            sent[i, idx] += val.astype(np.float64)
            fed[i] += float(F32(lr)) * o.get_grad(i).astype(np.float64)
        o.aggregate()
        o.apply_delayed()
    for i in range(w.n):
        assert np.abs(sent[i] + o.get_error(i) - fed[i]).max() <= 10 * 2.0 ** -22 * np.abs(fed).max()


def test_random_k_with_k_equal_d_is_dsgd(oracle_mod):
    o, w, lam, xstar, x0 = make(oracle_mod, 1200, 4, 0, seed=22)
    lr = 0.05
    x = x0.copy()
    for t in range(8):
        o.grad()
        gs = [o.get_grad(i) for i in range(w.n)]
        o.ef_compress(1.0, lr)
        o.aggregate()
        o.apply_delayed()
        acc = np.zeros(w.d, dtype=F32)
        for i in range(w.n):
            acc = acc + F32(lr) * gs[i]
            assert np.all(bits(o.get_error(i)) == 0)
        x = x - acc / F32(w.n)
        assert np.array_equal(bits(o.get_model()), bits(x))


def test_random_k_is_unbiased_up_to_the_ratio(oracle_mod):
    # E[C(p)] = (k/d) p: average the compressed vector over many independent draws
    d, k, draws = 400, 40, 4000
    p = workloads.random_vector(3, d, "normal").astype(np.float64)
    acc = np.zeros(d)
    for t in range(draws):
        idx = oracle_mod.randk_indices(9, t, 0, d, k)
        acc[idx] += p[idx]
    est = acc / draws
    sd = np.abs(p) * np.sqrt((k / d) * (1 - k / d) / draws)
    assert np.all(np.abs(est - (k / d) * p) <= 5 * sd + 1e-12)
