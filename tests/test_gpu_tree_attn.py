"""GPU parity of ss_spec_verify_attn on draft trees (ss_batch.tree_mask) against the CPU oracle."""
import numpy as np
import pytest

from paper_2604_09562_amd import binding, synth
from tests.test_gpu_attn import check, run_gpu

pytestmark = pytest.mark.gpu

TINY, LLAMA8B, RAGGED, LONG, FP8_70B = synth.CONFIGS


def test_tiny_fp32_tree(oracle):
    for seed in range(3):
        inp = synth.make_attention_inputs(TINY.scaled(depth=("uniform", 0, 8)), seed=seed, tree=True)
        assert check(inp, oracle, label=f"tiny tree seed {seed}") < 1e-4


@pytest.mark.parametrize("path", [0, 1])
@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("hq,hkv", [(8, 8), (8, 4), (16, 4), (16, 2)])
def test_small_shapes_all_groupings_tree(oracle, path, kv_dtype, hq, hkv):
    cfg = LLAMA8B.scaled(batch=6, num_q_heads=hq, num_kv_heads=hkv, kv_dtype=kv_dtype,
                         ctx=("uniform", 9, 700), depth=("uniform", 0, 8))
    inp = synth.make_attention_inputs(cfg, seed=hq + hkv, tree=True)
    binding.ss_set_option("attn_path", path)
    try:
        check(inp, oracle, label=f"tree {kv_dtype} {hq}/{hkv} path {path}")
    finally:
        binding.ss_set_option("attn_path", 0)


def test_edge_lengths_tree(oracle):
    # new tokens only, new tokens straddling a block boundary at every offset, exact block multiples
    kv_len = np.array([1, 9, 16, 17, 18, 19, 20, 21, 22, 23, 24, 25, 32, 5, 48, 255, 256, 257], np.int32)
    depth = np.array([0, 8, 3, 8, 8, 8, 8, 8, 8, 8, 8, 8, 0, 4, 8, 2, 8, 7], np.int32)
    for cfg in (LLAMA8B, FP8_70B):
        inp = synth.make_attention_inputs(cfg.scaled(batch=len(kv_len)), seed=3, kv_len=kv_len, depth=depth, tree=True)
        check(inp, oracle, label=f"tree edge lengths {cfg.kv_dtype}")


def test_star_and_chain_shapes(oracle):
    # a star (every draft a child of the root: rows see only themselves among the drafts) and a chain
    # written as a tree, which must reproduce the chain call bit for bit
    cfg = LLAMA8B.scaled(batch=5, ctx=("uniform", 50, 900), depth=("uniform", 0, 8))
    inp = synth.make_attention_inputs(cfg, seed=6)
    n = np.diff(inp["q_indptr"])
    star = dict(inp)
    star["tree_parent"] = np.concatenate([[-1] + [0] * (k - 1) for k in n]).astype(np.int32)
    star["tree_mask"] = np.concatenate([[1] + [1 | (1 << i) for i in range(1, k)] for k in n]).astype(np.uint32)
    check(star, oracle, label="star")
    chain = dict(inp)
    chain["tree_mask"] = np.concatenate([[(2 << i) - 1 for i in range(k)] for k in n]).astype(np.uint32)
    o_tree, l_tree = run_gpu(chain)
    o_chain, l_chain = run_gpu(inp)
    assert np.array_equal(o_tree, o_chain) and np.array_equal(l_tree, l_chain)


def test_partition_count_invariance_tree(oracle):
    cfg = LLAMA8B.scaled(batch=5, ctx=("uniform", 300, 3000), depth=("uniform", 0, 8))
    inp = synth.make_attention_inputs(cfg, seed=2, tree=True)
    try:
        for waves in (4, 64, 0):
            binding.ss_set_option("attn_waves", waves)
            check(inp, oracle, label=f"tree waves {waves}")
    finally:
        binding.ss_set_option("attn_waves", 0)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("cfg,max_q_len", [(LLAMA8B, 5), (RAGGED, 9), (FP8_70B, 9)],
                         ids=["llama3_8b_b64", "ragged_b128", "llama70b_fp8_b96"])
def test_full_size_configs_whole_batch_tree(oracle, cfg, max_q_len):
    inp = synth.make_attention_inputs(cfg, seed=0, tree=True)
    check(inp, oracle, max_q_len=max_q_len, label=f"tree {cfg.name}")


def test_validate_names_a_bad_mask():
    cfg = LLAMA8B.scaled(batch=3, ctx=("fixed", (40, 50, 60)), depth=("fixed", 3))
    inp = synth.make_attention_inputs(cfg, seed=0, tree=True)
    binding.ss_set_option("validate", 1)
    try:
        for row, word in ((5, 0b0101), (6, 0b10111)):   # row 1 of request 1 without its own bit; a bit past 4 rows
            bad = dict(inp)
            bad["tree_mask"] = inp["tree_mask"].copy()
            bad["tree_mask"][row] = word
            d = binding.attention_to_device(bad)
            out, lse, ws = binding.alloc_attention_outputs(d)
            with pytest.raises(binding.SpecVerifyError, match="tree mask"):
                binding.ss_spec_verify_attn(d, out, lse, ws)
        d = binding.attention_to_device(inp)
        out, lse, ws = binding.alloc_attention_outputs(d)
        binding.ss_spec_verify_attn(d, out, lse, ws)
    finally:
        binding.ss_set_option("validate", 0)
