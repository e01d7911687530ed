"""Pins for the oracle's greedy acceptance walk over draft trees (CPU only)."""
import numpy as np
import pytest

from paper_2604_09562_amd import synth

TINY = synth.CONFIGS[0]


def _explicit(logits, parent, tokens):
    """One request from explicit float32 target rows, parent list (node 0 first) and draft tokens."""
    logits = np.asarray(logits, dtype=np.float32)
    n, V = logits.shape
    return dict(batch=1, vocab=V, row_stride=V, logit_dtype="f32", total_rows=n,
                q_indptr=np.array([0, n], np.int32), target_logits=np.ascontiguousarray(logits),
                draft_tokens=np.asarray(tokens, np.int32), tree_parent=np.asarray(parent, np.int32))


def test_hand_worked_tree(oracle):
    # Vocabulary of 5.  Tree: 0 -> {1, 2, 3}; 2 -> {4, 5}; 4 -> {6}.
    # Row argmaxes: node0: 3, node2: 1 (tie between tokens 1 and 4 -> lowest index), node4: 0, node5: 2.
    rows = np.zeros((7, 5), np.float32)
    rows[0, 3] = 2.0
    rows[1, 0] = 9.0                  # node 1 is never reached: its row must not matter
    rows[2, 1] = rows[2, 4] = 1.5
    rows[3, 2] = 9.0
    rows[4, 0] = 0.5
    rows[5, 2] = 1.0
    rows[6, 4] = 3.0
    parent = [-1, 0, 0, 0, 2, 2, 4]
    # tokens of nodes 1..6: node1 wrong (2), node2 right (3), node3 right too but higher-numbered,
    # node4 right (1), node5 = 4 (the tied maximum's higher index: not the argmax), node6 wrong (1, needs 0)
    r = oracle.tree_accept_greedy(_explicit(rows, parent, [2, 3, 3, 1, 4, 1]))
    assert r["accepted_len"][0] == 2
    assert r["accepted_nodes"][0].tolist() == [2, 4] + [-1] * 18
    assert r["out_tokens"][0].tolist() == [3, 1, 0] + [-1] * 18
    # make node 6 right as well: the walk reaches a leaf and emits the leaf row's argmax as the bonus token
    r = oracle.tree_accept_greedy(_explicit(rows, parent, [2, 3, 3, 1, 4, 0]))
    assert r["accepted_len"][0] == 3
    assert r["accepted_nodes"][0].tolist()[:4] == [2, 4, 6, -1]
    assert r["out_tokens"][0].tolist()[:5] == [3, 1, 0, 4, -1]
    # nothing matches at the root: only the root's own next token comes out
    r = oracle.tree_accept_greedy(_explicit(rows, parent, [2, 0, 1, 1, 4, 0]))
    assert r["accepted_len"][0] == 0 and r["out_tokens"][0].tolist()[:2] == [3, -1]


def test_chain_trees_equal_the_chain_walk(oracle):
    cfg = TINY.scaled(batch=40, depth=("uniform", 0, 8), sigma_draft=("fixed", 0.3))
    inp = synth.make_accept_inputs(cfg, seed=5, greedy=True)
    ref = oracle.spec_accept(inp, greedy=True)
    assert 0 < ref["accepted_len"].mean() < inp["depth"].mean(), "the draw must mix accepts and rejects"
    as_tree = dict(inp)
    as_tree["tree_parent"] = np.concatenate([np.arange(-1, k) for k in inp["depth"]]).astype(np.int32)
    got = oracle.tree_accept_greedy(as_tree)
    assert np.array_equal(got["accepted_len"], ref["accepted_len"])
    assert np.array_equal(got["out_tokens"], ref["out_tokens"])
    for b, n in enumerate(got["accepted_len"]):
        assert got["accepted_nodes"][b].tolist() == list(range(1, n + 1)) + [-1] * (20 - n)


@pytest.mark.parametrize("logit_dtype", ["f32", "bf16"])
def test_output_is_plain_greedy_decoding_restricted_to_the_tree(oracle, logit_dtype):
    # Checked from the definition, without walking: the emitted tokens are the row maxima along the
    # reported path, the path is a parent chain whose draft tokens equal those maxima, no
    # lower-numbered sibling carried the same token, and the walk could not have gone on.
    cfg = TINY.scaled(batch=60, depth=("uniform", 0, 8), logit_dtype=logit_dtype, vocab=997)
    inp = synth.make_tree_accept_inputs(cfg, seed=3)
    r = oracle.tree_accept_greedy(inp)
    vals = synth.decode_storage(inp["target_logits"], logit_dtype)[:, :inp["vocab"]]
    lens = []
    for b in range(inp["batch"]):
        r0, k = int(inp["q_indptr"][b]), int(inp["depth"][b])
        par = inp["tree_parent"][r0:r0 + k + 1]
        tok = np.concatenate([[-1], inp["draft_tokens"][r0 - b:r0 - b + k]])
        n = int(r["accepted_len"][b])
        path = [0] + r["accepted_nodes"][b, :n].tolist()
        out = r["out_tokens"][b]
        assert np.all(r["accepted_nodes"][b, n:] == -1) and np.all(out[n + 1:] == -1)
        for j in range(n + 1):
            row = vals[r0 + path[j]]
            assert out[j] == int(np.flatnonzero(row == row.max())[0])
        for j in range(1, n + 1):
            c = path[j]
            assert par[c] == path[j - 1] and tok[c] == out[j - 1]
            assert not any(par[i] == path[j - 1] and tok[i] == out[j - 1] for i in range(1, c))
        assert not any(par[i] == path[n] and tok[i] == out[n] for i in range(1, k + 1))
        lens.append(n)
    assert 0.3 < np.mean(lens) and max(lens) >= 3 and min(lens) == 0


def test_bad_trees_rejected(oracle):
    rows = np.zeros((3, 4), np.float32)
    for parent in ([0, 0, 1], [-1, 1, 0], [-1, 0, 2], [-1, -1, 0]):
        with pytest.raises(ValueError):
            oracle.tree_accept_greedy(_explicit(rows, parent, [1, 2]))
