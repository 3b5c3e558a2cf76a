"""Pins for the oracle's DeCo rule (Algorithm 3, Remark on delta*(tau)) and the timing model
(Section 4.1 recurrence, Theorem 3 closed form and its error bound)."""
import math

import numpy as np
import pytest


def test_phi_degenerate_values(oracle_mod):
    # no compression: phi = 0 for every tau; no delay: phi = (1 - delta) / delta
    for tau in [0, 1, 7]:
        assert oracle_mod.phi(1.0, tau) == 0.0
    for delta in [0.5, 0.1, 0.001]:
        assert oracle_mod.phi(delta, 0) == pytest.approx((1 - delta) / delta, rel=1e-15)
    # worked value: delta = 0.5, tau = 2 -> 0.5 / (0.5 * 0.75^2)
    assert oracle_mod.phi(0.5, 2) == pytest.approx(1.0 / 0.5625, rel=1e-15)
    # phi grows with tau and shrinks with delta
    assert oracle_mod.phi(0.01, 4) > oracle_mod.phi(0.01, 3)
    assert oracle_mod.phi(0.02, 4) < oracle_mod.phi(0.01, 4)


def test_delta_star_reaches_t_comp(oracle_mod):
    # T_avg(tau, delta*(tau)) = T_comp whenever delta*(tau) > 0
    v_g, a, b, t_comp = 32 * 124e6, 1e8, 0.2, 0.25
    for tau in range(1, 12):
        ds = oracle_mod.delta_star(tau, v_g, a, b, t_comp)
        assert 0.0 <= ds <= 1.0
        if ds > 0:
            assert oracle_mod.t_avg_closed_form(tau, ds, v_g, a, b, t_comp) == pytest.approx(t_comp, rel=1e-12)
            # a larger ratio at the same tau costs time
            if ds < 1:
                assert oracle_mod.t_avg_closed_form(tau, min(1.0, ds * 1.5), v_g, a, b, t_comp) > t_comp
    assert oracle_mod.delta_star(0, v_g, a, b, t_comp) == 0.0


def brute_deco(v_g, a, b, t_comp):
    lo = math.ceil(b / t_comp)
    hi = math.ceil((b + v_g / a) / t_comp)
    best = None
    for tau in range(lo, hi + 1):                       # ascending, strict "<": smallest tau on ties
        delta = min((tau * t_comp - b) * a / v_g, t_comp * a / v_g, 1.0)
        if delta <= 0:
            continue
        phi = (1 - delta) / (delta * (1 - delta / 2) ** tau)
        if best is None or phi < best[0]:
            best = (phi, tau, delta)
    return best


def test_deco_matches_exhaustive_scan(oracle_mod):
    rng = np.random.default_rng(0)
    for _ in range(200):
        d = 10 ** rng.uniform(6, 9)
        v_g = 32 * d
        a = 10 ** rng.uniform(8, 10)
        b = rng.uniform(0.01, 0.3)
        t_comp = 10 ** rng.uniform(-2, 0)
        got = oracle_mod.deco(v_g, a, b, t_comp)
        want = brute_deco(v_g, a, b, t_comp)
        assert (got is None) == (want is None)
        if got:
            assert got[0] == want[1]
            assert got[1] == pytest.approx(want[2], rel=1e-12)


def test_deco_fast_network_returns_no_compression(oracle_mod):
    # bandwidth so high that the whole gradient fits in one compute slot: delta = 1, phi = 0,
    # and the smallest tau with delta = 1 wins
    v_g, a, b, t_comp = 32e6, 1e12, 0.05, 0.1
    tau, delta = oracle_mod.deco(v_g, a, b, t_comp)
    assert delta == 1.0
    assert tau == math.ceil((b + v_g / a) / t_comp)


@pytest.mark.parametrize("tau,delta,a,b,t_comp", [
    (0, 1.0, 1e9, 0.1, 0.3),      # D-SGD: serial compute + latency + transfer
    (2, 0.01, 1e8, 0.2, 0.25),    # compute bound
    (1, 0.5, 1e8, 0.2, 0.05),     # transfer bound
    (3, 0.05, 1e8, 1.0, 0.1),     # latency bound
    (8, 0.001, 2e8, 0.3, 0.02),
])
def test_theorem3_against_recurrence(oracle_mod, tau, delta, a, b, t_comp):
    v_g = 32 * 124e6
    for E in [50, 500, 5000]:
        rec = oracle_mod.t_avg_recurrence(tau, delta, v_g, a, b, t_comp, E)
        cf = oracle_mod.t_avg_closed_form(tau, delta, v_g, a, b, t_comp)
        bound = (b + min(t_comp, delta * v_g / a)) / E
        assert abs(rec - cf) <= bound * (1 + 1e-9) + 1e-15
    # tau = 0: every iteration is compute, then transfer, then latency, in series
    if tau == 0:
        assert cf == pytest.approx(t_comp + b + delta * v_g / a, rel=1e-12)


@pytest.mark.parametrize("delta,a,b,t_comp", [(1.0, 1e9, 0.1, 0.3), (0.02, 3e8, 0.25, 0.05), (0.5, 1e8, 0.0, 0.2)])
def test_recurrence_in_the_cases_that_can_be_worked_by_hand(oracle_mod, delta, a, b, t_comp):
    """Where the pipeline of Section 4.1 cannot overlap anything its completion time is a plain sum:
    a single iteration computes, transfers and waits out the latency, whatever tau is; and with
    tau = 0 every iteration waits for the one before it to arrive, so E iterations take E times
    that (the latency of the last message included)."""
    v_g = 32 * 11.7e6
    serial = t_comp + delta * v_g / a + b
    for tau in (0, 1, 5):
        assert oracle_mod.t_avg_recurrence(tau, delta, v_g, a, b, t_comp, 1) == pytest.approx(serial, rel=1e-12)
    for E in (2, 3, 50, 777):
        assert oracle_mod.t_avg_recurrence(0, delta, v_g, a, b, t_comp, E) == pytest.approx(serial, rel=1e-12)
    # tau = 1, two iterations, by hand: the second computation starts when the first ends (the
    # message it would wait for dates from before the start), its transfer when both the first
    # transfer and the second computation are over
    xfer = delta * v_g / a
    tm1 = t_comp + xfer
    tm2 = xfer + max(tm1, 2 * t_comp)
    assert oracle_mod.t_avg_recurrence(1, delta, v_g, a, b, t_comp, 2) == pytest.approx((tm2 + b) / 2, rel=1e-12)
