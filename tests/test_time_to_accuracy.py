"""Host logic of the time-to-accuracy study (no GPU): the four (tau, delta) strategies and their
iteration times under the pipeline model of Section 4.1 / Theorem 3."""
import math

import pytest

from paper_2507_17346_amd import time_to_accuracy as tta


def test_strategies_and_their_iteration_times():
    # V_g / a = 0.32 s, b = 0.1 s, T_comp = 0.02 s
    net = tta.Network(32.0 * 200_000, 20e6, 0.1, 0.02)
    ss = {s.name: s for s in tta.strategies(net, 16)}
    assert (ss["D-SGD"].tau, ss["D-SGD"].delta) == (0, 1.0)
    assert ss["compression only"].tau == 0
    assert ss["compression only"].delta == pytest.approx(0.02 * 20e6 / (32.0 * 200_000))
    assert (ss["delay only"].tau, ss["delay only"].delta) == (16, 1.0)          # ceil(0.42 / 0.02) = 21, clamped
    # DeCo: the smallest staleness that lets the bandwidth-matched ratio through (Algorithm 3)
    assert ss["DeCo"].tau == 6 and ss["DeCo"].delta == pytest.approx(0.0625)
    # iteration times: nothing hidden for tau = 0; bandwidth-bound without compression;
    # T_comp once both are matched (Theorem 3's three regimes)
    assert tta.t_avg(net, ss["D-SGD"]) == pytest.approx(0.02 + 0.32 + 0.1, rel=1e-3)
    assert tta.t_avg(net, ss["compression only"]) == pytest.approx(0.02 + 0.02 + 0.1, rel=1e-3)
    assert tta.t_avg(net, ss["delay only"]) == pytest.approx(0.32, rel=2e-2)
    assert tta.t_avg(net, ss["DeCo"]) == pytest.approx(0.02, rel=2e-2)
    assert set(ss) == {"D-SGD", "compression only", "delay only", "DeCo"}


def test_a_fast_network_needs_neither():
    # a gradient crosses in a tenth of T_comp and the latency is negligible: DeCo asks for no compression
    net = tta.Network(32.0 * 1000, 16e6, 1e-4, 0.02)
    ss = {s.name: s for s in tta.strategies(net, 16)}
    assert ss["DeCo"].delta == 1.0 and ss["DeCo"].tau <= 2
    assert ss["compression only"].delta == 1.0
    assert math.isclose(tta.t_avg(net, ss["DeCo"]), 0.02, rel_tol=0.15)
