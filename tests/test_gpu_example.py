"""The end-to-end example must run as shipped, for chains and for trees, and keep its books."""
import numpy as np
import pytest

from paper_2604_09562_amd import example

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("tree,sample", [(False, False), (True, False), (True, True)], ids=["chain", "tree", "tree_sampled"])
def test_example_decode_lane(tree, sample):
    r = example.run(steps=4, batch=5, layers=3, tree=tree, vocab=4096, seed=3, verbose=False, sample=sample)
    assert 0 <= r["chosen"] < 4
    assert r["emitted"] >= 4 * 5                       # every request emits at least one token per step
    # every emitted token but the one still in flight has become a valid cache position
    assert int((r["kv_len"] - r["start_len"]).sum()) == r["emitted"]
    assert np.all(r["depths"] >= 0) and np.all(r["depths"] <= 20)
