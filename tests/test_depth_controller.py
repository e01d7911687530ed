"""The library's depth controller (host arithmetic behind the C ABI) against the oracle's, step by step.

Both run in IEEE double; the sums over the flow vector are taken in the same index order, so real
outputs are compared to 1e-12 relative and the integer outputs (micro-batch size, depth) exactly.
Runs without a GPU: the controller launches nothing.
"""
import numpy as np
import pytest

from oracle.depth_controller import DepthController
from paper_2604_09562_amd import binding


def test_matches_oracle_over_random_metric_streams():
    rng = np.random.default_rng(12)
    for trial in range(20):
        st = binding.ss_depth_init()
        h = int(rng.integers(1, 33))
        st.h = h
        st.gamma = float(rng.uniform(1, 10))
        st.d_base = float(rng.uniform(1, 9))
        st.tau_target = float(rng.uniform(50, 1000))
        st.tau_recent = 123.0
        ref = DepthController(h=h, d_base=st.d_base, gamma=st.gamma, tau_target=st.tau_target, tau_recent=123.0)
        for step in range(60):
            a, l, t = float(rng.uniform(0, 1)), float(rng.uniform(0, 1.2)), float(rng.choice([0.0, 0.5, 80.0, 400.0, 2000.0]))
            got = binding.ss_depth_update(st, a, l, t)
            want = ref.update(a, l, t)
            assert got[0] == pytest.approx(want[0], rel=1e-12)
            assert got[1] == want[1] and got[3] == want[3]
            assert got[2] == pytest.approx(want[2], rel=1e-12)
            assert st.tau_recent == pytest.approx(ref.tau_recent, rel=1e-12)
            assert st.idx == ref.idx
            assert list(st.f[:h]) == pytest.approx(ref.f, rel=1e-12, abs=1e-15)


def test_defaults_are_the_papers():
    st = binding.ss_depth_init()
    assert (st.h, st.d_base, st.gamma, st.d_min, st.d_max, st.tau_target, st.tau_recent) == (10, 5.0, 5.0, 2.0, 20.0, 400.0, 0.0)
    d, b, tp, k = binding.ss_depth_update(st, 0.8, 0.25, 200.0)
    assert d == pytest.approx(5.48) and b == 14 and k == 5 and tp == pytest.approx(280.0)


def test_bad_arguments():
    st = binding.ss_depth_init()
    st.h = 0
    with pytest.raises(binding.SpecVerifyError):
        binding.ss_depth_update(st, 0.5, 0.0, 100.0)
    st = binding.ss_depth_init()
    with pytest.raises(binding.SpecVerifyError):
        binding.ss_depth_update(st, float("nan"), 0.0, 100.0)
