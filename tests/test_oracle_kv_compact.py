"""Pins of the oracle's cache compaction after acceptance over a draft tree (CPU only).

Checked against things the oracle's compaction code did not produce: the decoded token sequence of
the cache before the call (through the test helper's own paged gather and torch's decoders), torch's
float8 cast for the rescaled bytes, and the attention oracle's tree rows.
"""
import numpy as np
import pytest
import torch

from paper_2604_09562_amd import synth
from tests.helpers import gather_kv

TINY, LLAMA8B, RAGGED, LONG, FP8_70B = synth.CONFIGS
NODES = 20   # row width of accepted_nodes: the largest draft depth


def random_paths(inp, seed):
    """A random root path of every request's tree: (accepted_nodes [B][8], accepted_len [B])."""
    rng = np.random.default_rng(seed)
    B = inp["batch"]
    nodes = np.full((B, NODES), -1, np.int32)
    n = np.zeros(B, np.int32)
    for b in range(B):
        r0, q_len = int(inp["q_indptr"][b]), int(inp["q_indptr"][b + 1] - inp["q_indptr"][b])
        node = int(rng.integers(0, q_len))
        path = []
        while node > 0:
            path.append(node)
            node = int(inp["tree_parent"][r0 + node])
        path.reverse()
        n[b] = len(path)
        nodes[b, :len(path)] = path
    return nodes, n


def copy_batch(inp):
    out = dict(inp)
    for name in ("k_cache", "v_cache", "kv_len"):
        out[name] = inp[name].copy()
    return out


@pytest.mark.parametrize("kv_dtype", ["f32", "bf16"])
def test_compacted_cache_holds_context_then_path(oracle, kv_dtype):
    cfg = LLAMA8B.scaled(batch=24, num_q_heads=8, num_kv_heads=2, head_dim=64, kv_dtype=kv_dtype,
                         q_dtype="f32" if kv_dtype == "f32" else "bf16", ctx=("uniform", 9, 120), depth=("uniform", 0, 8))
    pre = synth.make_attention_inputs(cfg, seed=5, tree=True)
    nodes, n = random_paths(pre, 1)
    assert any(nodes[b, j] != j + 1 for b in range(24) for j in range(n[b])), "no path needs a move"
    post = copy_batch(pre)
    oracle.kv_compact(post, nodes, n)
    post["kv_len"] = oracle.kv_commit(pre["q_indptr"], n, pre["kv_len"])
    touched = {"k": np.zeros(pre["k_cache"].shape[:3], bool), "v": np.zeros(pre["k_cache"].shape[:3], bool)}
    for b in range(24):
        q_len = int(pre["q_indptr"][b + 1] - pre["q_indptr"][b])
        P = int(pre["kv_len"][b]) - q_len
        assert post["kv_len"][b] == P + 1 + n[b]
        for kind in "kv":
            before, after = gather_kv(pre, b, kind), gather_kv(post, b, kind)
            want = np.concatenate([before[:P + 1]] + [before[P + a:P + a + 1] for a in nodes[b, :n[b]]])
            assert np.array_equal(after, want)
            for j in range(1, n[b] + 1):
                pos = P + j
                touched[kind][pre["block_table"][b, pos // 16], :, pos % 16] = True
    # nothing but the destination slots changed, rejected slots and unreferenced blocks included
    for kind, name in (("k", "k_cache"), ("v", "v_cache")):
        same = pre[name].view(np.uint8).reshape(pre[name].shape[:3] + (-1,)) == \
            post[name].view(np.uint8).reshape(pre[name].shape[:3] + (-1,))
        assert np.all(same.all(axis=-1) | touched[kind])


def test_fp8_moves_across_blocks_are_rescaled_like_the_library_cast(oracle):
    # new tokens straddle a block boundary at every offset, so some moves change block (and scale)
    kv_len = np.tile(np.arange(17, 33, dtype=np.int32), 8)
    depth = np.full(128, 8, np.int32)
    cfg = FP8_70B.scaled(batch=128, num_q_heads=8, num_kv_heads=2)
    pre = synth.make_attention_inputs(cfg, seed=2, kv_len=kv_len, depth=depth, tree=True)
    nodes, n = random_paths(pre, 3)
    post = copy_batch(pre)
    oracle.kv_compact(post, nodes, n)
    crossed = 0
    for b in range(128):
        P = int(kv_len[b]) - 9
        for j in range(1, n[b] + 1):
            a = int(nodes[b, j - 1])
            bs_, bd = pre["block_table"][b, (P + a) // 16], pre["block_table"][b, (P + j) // 16]
            for name, sc in (("k_cache", "k_scale"), ("v_cache", "v_scale")):
                src = pre[name][bs_, :, (P + a) % 16, :]
                got = post[name][bd, :, (P + j) % 16, :]
                if a == j or bs_ == bd:
                    assert np.array_equal(got, src)
                    continue
                crossed += 1
                x = torch.from_numpy(src.copy()).view(torch.float8_e4m3fn).to(torch.float32)
                y = x * torch.from_numpy(pre[sc][bs_])[:, None] / torch.from_numpy(pre[sc][bd])[:, None]
                want = y.clamp(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
                assert np.array_equal(got, want)
    assert crossed >= 8
    assert np.array_equal(post["k_scale"], pre["k_scale"]) and np.array_equal(post["v_scale"], pre["v_scale"])


def test_a_chain_path_moves_nothing(oracle):
    cfg = LLAMA8B.scaled(batch=6, num_q_heads=8, num_kv_heads=2, ctx=("uniform", 9, 80), depth=("uniform", 0, 8))
    pre = synth.make_attention_inputs(cfg, seed=1, tree=True)
    n = (pre["depth"] // 2).astype(np.int32)
    nodes = np.full((6, NODES), -1, np.int32)
    for b in range(6):
        nodes[b, :n[b]] = np.arange(1, n[b] + 1)
    post = copy_batch(pre)
    oracle.kv_compact(post, nodes, n)
    assert np.array_equal(post["k_cache"], pre["k_cache"]) and np.array_equal(post["v_cache"], pre["v_cache"])


def test_tree_row_before_equals_chain_row_after(oracle):
    # The deepest accepted node's attention output over the tree (ancestor mask) must equal the last
    # row of a chain verify over the compacted, committed cache: same keys and values in the same order.
    cfg = LLAMA8B.scaled(batch=10, num_q_heads=8, num_kv_heads=2, ctx=("uniform", 9, 100), depth=("uniform", 1, 8))
    pre = synth.make_attention_inputs(cfg, seed=7, tree=True)
    nodes, n = random_paths(pre, 5)
    o_tree, l_tree = oracle.verify_attn(pre)
    post = copy_batch(pre)
    oracle.kv_compact(post, nodes, n)
    post["kv_len"] = oracle.kv_commit(pre["q_indptr"], n, pre["kv_len"])
    del post["tree_mask"], post["tree_parent"]
    rows = [[int(pre["q_indptr"][b])] + [int(pre["q_indptr"][b]) + int(a) for a in nodes[b, :n[b]]] for b in range(10)]
    post["q_indptr"] = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
    post["total_rows"] = int(post["q_indptr"][-1])
    flat = np.concatenate(rows)
    post["q"] = np.ascontiguousarray(pre["q"][flat])
    o_chain, l_chain = oracle.verify_attn(post)
    assert np.array_equal(o_chain, o_tree[flat]) and np.array_equal(l_chain, l_tree[flat])


def test_bad_paths_rejected(oracle):
    cfg = LLAMA8B.scaled(batch=2, num_q_heads=8, num_kv_heads=2, ctx=("fixed", (40, 50)), depth=("fixed", 4))
    pre = synth.make_attention_inputs(cfg, seed=0, tree=True)
    for path, n in (([2, 1], 2), ([5], 1), ([1, 1], 2), ([0], 1)):
        nodes = np.full((2, NODES), -1, np.int32)
        nodes[1, :len(path)] = path
        with pytest.raises(ValueError):
            oracle.kv_compact(copy_batch(pre), nodes, np.array([0, n], np.int32))
    with pytest.raises(ValueError):
        oracle.kv_compact(copy_batch(pre), np.full((2, NODES), -1, np.int32), np.array([0, 5], np.int32))
