"""Host-side DeCo pieces of the library (Algorithm 3, Theorem 3, the look-up table of Section 4.5)
against the oracle's independent versions and against what the paper fixes; no GPU needed."""
import math

import numpy as np
import pytest

from paper_2507_17346_amd import binding

V_G = 32 * 124e6


def test_phi_and_timing_model_match_oracle(oracle_mod):
    rng = np.random.default_rng(3)
    for _ in range(300):
        delta = float(10 ** rng.uniform(-4, 0))
        tau = int(rng.integers(0, 17))
        a = 10 ** rng.uniform(8, 10)
        b = rng.uniform(0.01, 1.0)
        t_comp = 10 ** rng.uniform(-2, 0)
        assert binding.phi(delta, tau) == pytest.approx(oracle_mod.phi(delta, tau), rel=1e-13)
        assert binding.t_avg_model(tau, delta, V_G, a, b, t_comp) == pytest.approx(
            oracle_mod.t_avg_closed_form(tau, delta, V_G, a, b, t_comp), rel=1e-13)
        for E in (1, 7, 50, 333):
            assert binding.t_avg_simulate(tau, delta, V_G, a, b, t_comp, E) == pytest.approx(
                oracle_mod.t_avg_recurrence(tau, delta, V_G, a, b, t_comp, E), rel=1e-12)
    assert binding.phi(1.0, 5) == 0.0
    assert math.isnan(binding.phi(0.0, 1)) and math.isnan(binding.phi(1.5, 1))


def test_simulation_stays_within_theorem3_bound():
    for tau, delta, a, b, t_comp in [(0, 1.0, 1e9, 0.1, 0.3), (2, 0.01, 1e8, 0.2, 0.25),
                                     (1, 0.5, 1e8, 0.2, 0.05), (3, 0.05, 1e8, 1.0, 0.1)]:
        for E in (50, 500):
            sim = binding.t_avg_simulate(tau, delta, V_G, a, b, t_comp, E)
            model = binding.t_avg_model(tau, delta, V_G, a, b, t_comp)
            assert abs(sim - model) <= (b + min(t_comp, delta * V_G / a)) / E * (1 + 1e-9)


def test_lut_matches_oracle_and_section_4_5(oracle_mod):
    b, t_comp, points = 0.2, 0.25, 20            # "like 20 points"
    a_min, a_max = 0.5e8, 2.0e8
    lut = binding.DecoLut(V_G, a_min, a_max, points, b, t_comp)
    table = oracle_mod.lut_build(V_G, a_min, a_max, points, b, t_comp)
    # pre-computation: every entry is the online decision at its sample bandwidth
    for a_i, entry in table:
        got = lut.query(a_i)
        assert got[2] is True
        assert (got[0], pytest.approx(got[1], rel=1e-12)) == oracle_mod.deco(V_G, a_i, b, t_comp) == entry
    # runtime lookup: nearest sample point inside the range, online computation outside
    rng = np.random.default_rng(4)
    step = (a_max - a_min) / (points - 1)
    for a in np.concatenate([rng.uniform(a_min, a_max, 200), [a_min, a_max, a_min + 0.49 * step, a_min + 0.51 * step]]):
        got = lut.query(float(a))
        want = oracle_mod.lut_query(table, V_G, b, t_comp, float(a))
        assert got[2] is True and want[2] is True
        assert got[0] == want[0] and got[1] == pytest.approx(want[1], rel=1e-12)
        nearest = table[int(round((a - a_min) / step))][1]
        assert (got[0], pytest.approx(got[1], rel=1e-12)) == nearest
    for a in [a_min * 0.5, a_max * 1.5, 1e6, 1e11]:
        got = lut.query(a)
        want = oracle_mod.deco(V_G, a, b, t_comp)
        assert got[2] is False
        assert got[0] == want[0] and got[1] == pytest.approx(want[1], rel=1e-12)
    # the rounding error of the table is what the scheme accepts: at most half a step in bandwidth
    lut.close()
    import ctypes as C
    lib = binding.load()
    h = C.c_void_p()
    assert lib.ddef_lut_build(V_G, 2e8, 1e8, 20, b, t_comp, C.byref(h)) == binding.EINVAL
    assert lib.ddef_lut_build(V_G, 1e8, 2e8, 1, b, t_comp, C.byref(h)) == binding.EINVAL
    assert lib.ddef_lut_destroy(None) == binding.EINVAL


def test_non_iid_objective_matches_oracle(oracle_mod):
    rng = np.random.default_rng(7)
    for _ in range(300):
        v_g = 32 * 10 ** rng.uniform(6, 9)
        a = 10 ** rng.uniform(8, 10)
        b = rng.uniform(0.01, 0.3)
        t_comp = 10 ** rng.uniform(-2, 0)
        got, want = binding.deco_noniid(v_g, a, b, t_comp), oracle_mod.deco_noniid(v_g, a, b, t_comp)
        assert (got is None) == (want is None)
        if got:
            assert got[0] == want[0] and got[1] == pytest.approx(want[1], rel=1e-12)
        delta, tau = float(10 ** rng.uniform(-4, 0)), int(rng.integers(0, 17))
        assert binding.phi_prime(delta, tau) == pytest.approx(oracle_mod.phi_prime(delta, tau), rel=1e-13)
    assert binding.phi_prime(1.0, 3) == 0.0 and math.isnan(binding.phi_prime(0.0, 3))
