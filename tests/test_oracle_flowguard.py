"""Pins of the router oracle against Section 3.2 (Eq. 1-4, Algorithm 2): numbers worked by hand."""
import pytest

from oracle import flowguard as fg


def test_score_by_hand():
    # 0.4*0.5 + 0.1*(1-0.2) + 0.3*(1-4/16) + 0.2*(1-0.25) = 0.2 + 0.08 + 0.225 + 0.15
    assert fg.score(0.5, 0.2, 4, 0.25, 16) == pytest.approx(0.655)
    assert fg.score(1.0, 0.0, 0, 0.0, 16) == pytest.approx(1.0)       # the weights sum to one
    assert fg.score(0.0, 1.0, 16, 1.0, 16) == pytest.approx(0.0)
    assert fg.score(0.0, 1.0, 400, 1.0, 16) == pytest.approx(0.0)     # queue term clipped at a full queue


def test_overload_by_hand():
    assert fg.overload_score(0.25, 4, 16) == pytest.approx(0.75)      # 0.25 + 2*4/16: under 0.85
    assert fg.overload_score(0.35, 4, 16) == pytest.approx(0.85)      # not above the threshold: still eligible
    assert fg.select([(0.0, 0.35, 4, 0.0, False)], 16) == 0
    assert fg.overload_score(0.40, 4, 16) > 0.85


def test_selection_branches():
    ok_low = (0.1, 0.2, 2, 0.5, False)      # score 0.04 + 0.08 + 0.2625 + 0.1 = 0.4825
    ok_high = (0.9, 0.2, 2, 0.5, False)     # 0.36 + 0.08 + 0.2625 + 0.1 = 0.8025
    over = (1.0, 0.9, 1, 0.0, False)        # omega = 0.9 + 0.125 > 0.85: excluded although its score is highest
    stale = (1.0, 0.0, 0, 0.0, True)
    assert fg.select([ok_low, ok_high, over, stale], 16) == 1
    assert fg.select([over, ok_low, stale], 16) == 1
    assert fg.select([ok_high, ok_high], 16) == 0                      # tie: lowest index
    # everyone overloaded or stale: minimum queue depth over all workers, lowest index on ties
    assert fg.select([(0, 0.9, 9, 0, False), (0, 0.9, 3, 0, False), (0, 0.9, 3, 0, True)], 16) == 1
    assert fg.select([(0, 0.0, 5, 0, True), (0, 0.0, 4, 0, True)], 16) == 1
