"""The library's router (host arithmetic behind the C ABI) against the oracle's selection, on random fleets
and on the hand-made branch cases.  Runs without a GPU."""
import numpy as np
import pytest

from oracle import flowguard as fg
from paper_2604_09562_amd import binding


def test_matches_oracle_on_random_fleets():
    rng = np.random.default_rng(5)
    hit = {"scored": 0, "fallback": 0}
    for trial in range(600):
        n = int(rng.integers(1, 12))
        q_max = float(rng.choice([8, 16, 64]))
        heavy = rng.random() < 0.4
        ws = [(float(rng.random()), float(rng.uniform(0.5, 1.0) if heavy else rng.random()),
               int(rng.integers(0, int(q_max) + 4)), float(rng.random()), bool(rng.random() < 0.2)) for _ in range(n)]
        want = fg.select(ws, q_max)
        assert binding.ss_route_select(ws, q_max) == want
        eligible = [w for w in ws if not w[4] and fg.overload_score(w[1], w[2], q_max) <= fg.TAU]
        hit["scored" if eligible else "fallback"] += 1
    assert min(hit.values()) > 30, hit      # both branches were exercised


def test_custom_weights_threshold_and_ties():
    ws = [(0.9, 0.2, 2, 0.5, False), (0.1, 0.0, 0, 0.0, False)]
    assert binding.ss_route_select(ws, 16) == fg.select(ws, 16) == 0
    al = (0.0, 0.0, 0.0, 1.0)               # only the load term counts
    assert binding.ss_route_select(ws, 16, alpha=al) == fg.select(ws, 16, alpha=al) == 1
    assert binding.ss_route_select(ws, 16, tau=0.1) == fg.select(ws, 16, tau=0.1) == 1   # worker 0: 0.2 + 0.25 > 0.1
    same = [(0.5, 0.1, 1, 0.1, False)] * 3
    assert binding.ss_route_select(same, 16) == 0


def test_bad_arguments():
    with pytest.raises(binding.SpecVerifyError):
        binding.ss_route_select([(0, 0, 0, 0, False)], 0.0)
