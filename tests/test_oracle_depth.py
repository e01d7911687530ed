"""Pins of the depth-controller oracle against what Section 3.5 (Eq. 8-16, Algorithm 4) fixes:
closed forms worked out by hand, the saturation point of each factor, and a short hand-computed run."""
import math

import pytest

from oracle.depth_controller import DepthController


def test_first_update_closed_form():
    # from the zero state: delta = a, f = [a, 0, ...], mag = a/h, d = d_base + a * (a/h) * gamma * adj * scale
    c = DepthController()
    d, b, tp, k = c.update(a=0.8, l=0.25, t=200.0)
    want = 5.0 + 0.8 * (0.8 / 10) * 5.0 * (1 - 0.25) * (400.0 / 200.0)
    assert d == pytest.approx(want, abs=1e-15) and want == pytest.approx(5.48, abs=1e-12)
    assert b == math.floor(80 / want) == 14
    assert tp == pytest.approx(200.0 * 1.4) and c.tau_recent == pytest.approx(28.0)
    assert k == 5 and c.idx == 1 and c.f[0] == pytest.approx(0.8)


def test_hand_worked_three_steps():
    # h = 2 keeps the arithmetic short.  a = 0.5, 1.0, 0.0 with l = 0, t >= target (scale 1).
    c = DepthController(h=2, d_base=5.0, gamma=5.0)
    d1, *_ = c.update(0.5, 0.0, 400.0)     # delta = 0.5, f = [0.5, 0], mag = 0.25, d = 5 + 0.5*0.25*5 = 5.625
    assert d1 == pytest.approx(5.625)
    d2, *_ = c.update(1.0, 0.0, 400.0)     # mean f = 0.25, delta = 0.75, f = [0.5, 0.75], mag = 0.625, d = 5 + 1*0.625*5
    assert d2 == pytest.approx(8.125)
    d3, b3, _, k3 = c.update(0.0, 0.0, 400.0)   # mean f = 0.625, delta = -0.625, f = [-0.625, 0.75]; a = 0 -> d = d_base
    assert d3 == pytest.approx(5.0) and c.f == pytest.approx([-0.625, 0.75])
    assert b3 == 16 and k3 == 5


def test_factor_saturation_and_clipping():
    # load saturates at 0.9 -> adj 0.1; throughput at or above target -> scale 1; below 1 token/s -> scale tau_target
    for l, adj in ((0.0, 1.0), (0.5, 0.5), (0.9, 0.1), (1.0, 0.1), (7.0, 0.1)):
        c = DepthController()
        d, *_ = c.update(1.0, l, 400.0)
        assert d == pytest.approx(5.0 + 1.0 * 0.1 * 5.0 * adj)
    for t, scale in ((400.0, 1.0), (4000.0, 1.0), (100.0, 4.0), (1.0, 400.0), (0.0, 400.0)):
        c = DepthController(d_max=1e9)
        d, *_ = c.update(1.0, 0.0, t)
        assert d == pytest.approx(5.0 + 0.5 * scale)
    c = DepthController()                      # unclipped 5 + 0.5*400 = 205 -> d_max = 20, b_micro = 4, k = 20
    d, b, _, k = c.update(1.0, 0.0, 0.0)
    assert (d, b, k) == (20.0, 4, 20)
    c = DepthController(d_base=0.5)            # below d_min
    d, b, _, k = c.update(0.0, 0.0, 400.0)
    assert (d, b, k) == (2.0, 40, 2)
    assert DepthController(d_min=0.01, d_base=0.01, d_max=0.01).update(0.0, 0.0, 1.0)[1] == 8000
    assert DepthController(d_min=100, d_base=100, d_max=100, k_cap=1000).update(0.0, 0.0, 1.0)[1:] == (1, 1.0, 100)


def test_smoothing_closed_form():
    # constant metrics: tau_n = 0.9^n tau_0 + (1 - 0.9^n) * t (1 + a/2)
    c = DepthController(tau_recent=50.0)
    for n in range(1, 40):
        c.update(0.6, 0.3, 300.0)
        want = 0.9 ** n * 50.0 + (1 - 0.9 ** n) * 300.0 * 1.3
        assert c.tau_recent == pytest.approx(want, rel=1e-12)


def test_constant_acceptance_flow_dies_out():
    # With a constant acceptance rate the gradient is a - mean(f); for h = 1 it alternates a, 0, a, 0, ...
    c = DepthController(h=1)
    ds = [c.update(0.5, 0.0, 400.0)[0] for _ in range(4)]
    assert ds == pytest.approx([5 + 0.5 * 0.5 * 5, 5.0, 5 + 0.5 * 0.5 * 5, 5.0])
    # the circular write position wraps after h updates
    c = DepthController(h=3)
    for i in range(7):
        c.update(0.1 * i, 0.0, 400.0)
    assert c.idx == 7 % 3
