"""Pins of the oracle's sampled acceptance over draft trees (CPU only).

The walk is a chain of speculative-sampling steps against a changing residual; what fixes it is that
the emitted tokens must be distributed as plain sampling from the target rows.  That identity is
checked by exact integration over every draft-token assignment and every cell of every uniform, with
the breakpoints of the cells computed here in numpy (not taken from the oracle).
"""
import itertools

import numpy as np
import pytest

from paper_2604_09562_amd import synth
from tests.helpers import softmax64
from tests.test_oracle_accept import _batch, _cells

TINY = synth.CONFIGS[0]


def _tree_batch(lp, lq, parent, cases, T):
    """cases: list of (tokens of nodes 1..k, uniforms of nodes 1..k, u_s); one request per case."""
    k = len(parent) - 1
    B = len(cases)
    inp = _batch([lp] * B, [lq] * B, [c[0] for c in cases], [c[1] for c in cases], [c[2] for c in cases], [k] * B, T=T)
    inp["tree_parent"] = np.tile(np.asarray(parent, np.int32), B)
    return inp


def _model(parent, p, q):
    """Independent numpy model: the distribution every node is offered to, and the distribution the
    final token is drawn from when the walk stops at a node (all of its children rejected)."""
    k = len(parent) - 1
    offered, final = {}, {}
    for cur in range(k + 1):
        r = p[cur].copy()
        for c in range(cur + 1, k + 1):
            if parent[c] != cur:
                continue
            offered[c] = r.copy()
            res = np.maximum(r - q[c - 1], 0.0)
            r = res / res.sum()
        final[cur] = r
    return offered, final


@pytest.mark.parametrize("parent,V,T,seed", [([-1, 0, 0], 4, 1.0, 0), ([-1, 0, 0, 0], 3, 0.8, 1), ([-1, 0, 0, 1], 3, 1.2, 2),
                                             ([-1, 0, 1, 1], 3, 1.0, 3), ([-1, 0, 1, 0, 3], 3, 0.9, 4)])
def test_emitted_tokens_follow_the_target_by_exact_integration(oracle, parent, V, T, seed):
    rng = np.random.default_rng(seed)
    k = len(parent) - 1
    lp = rng.normal(0, 1.5, size=(k + 1, V)).astype(np.float32)
    # siblings are drawn from one proposal (the draft model's distribution at their parent)
    lq_par = (lp + rng.normal(0, 1.0, size=(k + 1, V))).astype(np.float32)
    lq = np.stack([lq_par[parent[c]] for c in range(1, k + 1)])
    p = np.stack([softmax64(r, T) for r in lp])
    q = np.stack([softmax64(r, T) for r in lq])
    offered, final = _model(parent, p, q)
    us_mid, us_wid = _cells(np.concatenate([np.cumsum(final[c]) / final[c].sum() for c in final]))
    cases, weights = [], []
    for xs in itertools.product(range(V), repeat=k):
        wx = np.prod([q[c - 1][xs[c - 1]] for c in range(1, k + 1)])
        cells = [_cells(np.array([offered[c][xs[c - 1]] / q[c - 1][xs[c - 1]]])) for c in range(1, k + 1)]
        for ui in itertools.product(*[range(len(c[0])) for c in cells]):
            wu = np.prod([cells[i][1][ui[i]] for i in range(k)])
            u_acc = [cells[i][0][ui[i]] for i in range(k)]
            for m, w in zip(us_mid, us_wid):
                cases.append((list(xs), u_acc, m))
                weights.append(wx * wu * w)
    weights = np.asarray(weights)
    assert abs(weights.sum() - 1.0) < 1e-4
    res = oracle.tree_accept_sample(_tree_batch(lp, lq, parent, cases, T))
    n, toks, nodes = res["accepted_len"], res["out_tokens"], res["accepted_nodes"]
    # first emitted token ~ p_0, whichever way it came about (an accepted child or the final draw)
    got = np.zeros(V)
    np.add.at(got, toks[:, 0], weights)
    assert np.max(np.abs(got - p[0])) < 2e-5, (got, p[0])
    # after any accepted node c (whatever came before), the next emitted token ~ p_c
    for c in range(1, k + 1):
        for pos in range(k):
            sel = (n > pos) & (nodes[:, min(pos, nodes.shape[1] - 1)] == c)
            if weights[sel].sum() < 1e-9:
                continue
            got = np.zeros(V)
            np.add.at(got, toks[sel, pos + 1], weights[sel])
            assert np.max(np.abs(got / weights[sel].sum() - p[c])) < 1e-4, (c, pos)
    # the reported paths are parent chains carrying the emitted tokens
    for b in range(0, len(cases), 97):
        prev = 0
        for j in range(n[b]):
            c = nodes[b, j]
            assert parent[c] == prev and toks[b, j] == cases[b][0][c - 1]
            prev = c


def test_chains_reduce_to_the_chain_rule(oracle):
    cfg = TINY.scaled(batch=200, vocab=300, depth=("uniform", 0, 8), sigma_draft=("fixed", 0.7))
    inp = synth.make_accept_inputs(cfg, seed=9)
    ref = oracle.spec_accept(inp)
    as_tree = dict(inp, tree_parent=np.concatenate([np.arange(-1, k) for k in inp["depth"]]).astype(np.int32))
    got = oracle.tree_accept_sample(as_tree)
    assert 0 < ref["accepted_len"].mean() < inp["depth"].mean()
    assert np.array_equal(got["accepted_len"], ref["accepted_len"])
    assert np.array_equal(got["out_tokens"], ref["out_tokens"])
    tested = ~np.isnan(got["ratio"])
    assert np.allclose(got["ratio"][tested], ref["ratio"][tested], rtol=1e-12)
    # drafts after the first rejection are never offered in a chain
    for b in range(inp["batch"]):
        d0, k, n = inp["q_indptr"][b] - b, inp["depth"][b], ref["accepted_len"][b]
        assert tested[d0:d0 + min(n + 1, k)].all() and not tested[d0 + min(n + 1, k):d0 + k].any()


def test_second_sibling_by_hand(oracle):
    # V = 3, p = (.5, .3, .2), q = (.2, .5, .3); both children of the root carry token 1.
    # Child 1: ratio .3/.5 = .6.  After its rejection r = max(0, p-q)/.3 = (1, 0, 0): child 2 (token 1) has
    # ratio 0 and is rejected whatever its uniform; the final residual stays (1,0,0) -> token 0.
    p, q = np.array([.5, .3, .2]), np.array([.2, .5, .3])
    lp = np.log(np.stack([p, p, p])).astype(np.float32)
    lq = np.log(np.stack([q, q])).astype(np.float32)
    cases = [([1, 1], [0.59, 0.0], 0.9), ([1, 1], [0.61, 0.0], 0.9), ([1, 0], [0.61, 0.99], 0.2)]
    res = oracle.tree_accept_sample(_tree_batch(lp, lq, [-1, 0, 0], cases, 1.0))
    assert res["accepted_len"].tolist() == [1, 0, 1]
    assert res["accepted_nodes"][:, 0].tolist() == [1, -1, 2]
    assert res["out_tokens"][1, 0] == 0                      # both rejected: drawn from (1, 0, 0)
    assert res["out_tokens"][2, 0] == 0                      # second sibling (token 0) accepted at ratio 1/.2 > 1
    assert res["ratio"][:2] == pytest.approx([0.6, np.nan], nan_ok=True, rel=1e-6)
    assert res["ratio"][2:4] == pytest.approx([0.6, 0.0], abs=1e-6)
    assert res["ratio"][5] == pytest.approx(5.0, rel=1e-5)
