"""GPU parity at draft depths beyond 8, up to the controller's d_max = 20 (Section 3.5, Eq. 13)."""
import numpy as np
import pytest
import torch

from paper_2604_09562_amd import binding, synth
from tests.test_gpu_attn import check
from tests.test_gpu_accept import compare as compare_accept
from tests.test_gpu_kv import run_and_compare as append_and_compare

pytestmark = pytest.mark.gpu

TINY, LLAMA8B, RAGGED, LONG, FP8_70B = synth.CONFIGS


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("hq,hkv,kmax,path", [(8, 8, 20, 2), (8, 4, 20, 2), (16, 4, 19, 2), (16, 4, 20, 2), (16, 2, 20, 2),
                                               (16, 2, 13, 2), (16, 2, 20, 1)],
                         ids=["g1", "g2", "g4_one_pass", "g4_two_passes", "g8_three_passes", "g8_two_passes", "g8_vector"])
def test_attention_up_to_depth_20(oracle, kv_dtype, hq, hkv, kmax, path):
    # path 2 demands the matrix-core kernel: up to 80 query rows per KV head in one pass, more in
    # several passes over windows of query tokens; path 1 is the vector kernel
    cfg = LLAMA8B.scaled(batch=7, num_q_heads=hq, num_kv_heads=hkv, kv_dtype=kv_dtype, ctx=("uniform", 30, 900))
    depth = np.array([kmax, 0, 9, 13, kmax, 8, 17][:7], np.int32)
    depth = np.minimum(depth, kmax)
    kv_len = np.array([21, 40, 333, 47, 900, 64, 129], np.int32)
    for tree in (False, True):
        inp = synth.make_attention_inputs(cfg, seed=hq + kmax, kv_len=kv_len, depth=depth, tree=tree)
        binding.ss_set_option("attn_path", path)
        try:
            check(inp, oracle, max_q_len=int(depth.max()) + 1, label=f"deep {kv_dtype} {hq}/{hkv} k<={kmax} tree={tree}")
        finally:
            binding.ss_set_option("attn_path", 0)


@pytest.mark.parametrize("greedy", [False, True])
def test_accept_up_to_depth_20(oracle, greedy):
    cfg = LLAMA8B.scaled(batch=12, vocab=20011, sigma_draft=("fixed", 0.25))
    depth = np.array([20, 0, 9, 13, 20, 8, 17, 1, 20, 12, 16, 19], np.int32)
    inp = synth.make_accept_inputs(cfg, seed=3, depth=depth, greedy=greedy, row_pad=(-20011) % 8)
    compare_accept(inp, oracle, greedy=greedy, label=f"deep accept greedy={greedy}")
    assert oracle.spec_accept(inp, greedy=greedy)["accepted_len"].max() > 8, "no request got past depth 8"


def test_append_and_tree_steps_up_to_depth_20(oracle):
    depth = np.array([20, 0, 9, 13, 20, 8, 17, 20], np.int32)
    kv_len = np.array([21, 40, 333, 47, 900, 64, 129, 60], np.int32)
    for cfg in (LLAMA8B.scaled(batch=8), FP8_70B.scaled(batch=8)):
        inp = synth.make_append_inputs(cfg, seed=1, kv_len=kv_len, depth=depth)   # 21 new tokens span three blocks
        append_and_compare(inp, oracle, f"deep append {cfg.kv_dtype}")
        # greedy tree acceptance and compaction on the same shapes
        acc_in = synth.make_tree_accept_inputs(cfg.scaled(vocab=4096), seed=2, depth=depth, hit=0.8)
        ref = oracle.tree_accept_greedy(acc_in)
        da = binding.accept_to_device({**acc_in, "draft_logits": None, "u_accept": None, "u_sample": None, "temperature": None})
        n_acc, toks, _, ws = binding.alloc_accept_outputs(da)
        nodes = torch.full((8, binding.SS_MAX_DEPTH), -77, dtype=torch.int32, device="cuda:0")
        binding.ss_spec_accept_tree_greedy(da, n_acc, toks, nodes, ws)
        torch.cuda.synchronize()
        assert np.array_equal(n_acc.cpu().numpy(), ref["accepted_len"]) and np.array_equal(toks.cpu().numpy(), ref["out_tokens"])
        assert np.array_equal(nodes.cpu().numpy(), ref["accepted_nodes"])
        d = binding.attention_to_device(inp)
        binding.ss_kv_compact(d, nodes, n_acc)
        torch.cuda.synchronize()
        oracle.kv_compact(inp, ref["accepted_nodes"], ref["accepted_len"])
        for name in ("k_cache", "v_cache"):
            assert np.array_equal(d[name].cpu().numpy().view(np.uint8), inp[name].view(np.uint8)), name


def test_unknown_row_bound_is_correct_for_every_grouping(oracle):
    # max_q_len = 0: the library must assume 21 rows per request; groups of 4 and 8 are then served in
    # two and three passes, the later ones finding no rows at these depths
    for hq, hkv in ((8, 8), (8, 4), (16, 4), (16, 2)):
        cfg = LLAMA8B.scaled(batch=4, num_q_heads=hq, num_kv_heads=hkv, ctx=("uniform", 30, 500), depth=("uniform", 0, 8))
        inp = synth.make_attention_inputs(cfg, seed=hq)
        check(inp, oracle, max_q_len=0, label=f"unknown bound {hq}/{hkv}")


def test_batches_larger_than_a_workgroup(oracle):
    # 300 requests: every per-request loop that strides by the workgroup size takes a second trip
    cfg = LLAMA8B.scaled(batch=300, vocab=2500, ctx=("uniform", 5, 90), depth=("uniform", 0, 8))
    inp = synth.make_append_inputs(cfg, seed=6)
    append_and_compare(inp, oracle, "300 requests: append")
    check(inp, oracle, label="300 requests: attention")
    binding.ss_set_option("validate", 1)
    try:
        check(inp, oracle, label="300 requests: attention, validated")
    finally:
        binding.ss_set_option("validate", 0)
    acc_in = synth.make_accept_inputs(cfg, seed=6, depth=inp["depth"], row_pad=(-2500) % 8)
    compare_accept(acc_in, oracle, label="300 requests: accept")
    d = binding.attention_to_device(inp)
    n = binding._to_dev(oracle.spec_accept(acc_in)["accepted_len"], "cuda:0")
    binding.ss_kv_commit(d["q_indptr"], n, d["kv_len"])
    torch.cuda.synchronize()
    assert np.array_equal(d["kv_len"].cpu().numpy(), oracle.kv_commit(inp["q_indptr"], n.cpu().numpy(), inp["kv_len"]))


def test_batch_beyond_the_plan_kernels_prefix_buffer(oracle):
    # more than 4096 requests: the plan kernel cannot hold the tile prefix in LDS and cuts the spans unweighted
    cfg = LLAMA8B.scaled(batch=4300, num_q_heads=8, num_kv_heads=2, ctx=("uniform", 3, 40), depth=("uniform", 0, 2))
    inp = synth.make_attention_inputs(cfg, seed=8)
    check(inp, oracle, label="4300 requests")


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("hq,hkv", [(8, 8), (8, 4), (16, 4), (16, 2)], ids=["g1", "g2", "g4", "g8"])
def test_tree_depth_20_tail_slots_stay_invisible(oracle, kv_dtype, hq, hkv):
    # 21 new tokens whose first one sits at ctx % 16 == 12: the last tile's last lane group starts 32
    # positions behind ctx, one past the mask word's last bit.  Those slots (and everything else past
    # kv_len) hold NaN; a row that saw them would come out NaN or mis-normalised.
    cfg = LLAMA8B.scaled(batch=6, num_q_heads=hq, num_kv_heads=hkv, kv_dtype=kv_dtype)
    kv_len = np.array([33, 49, 705, 65, 45, 34], np.int32)     # the first four have (kv_len - 21) % 16 == 12
    depth = np.array([20, 20, 20, 20, 20, 20], np.int32)
    inp = synth.make_attention_inputs(cfg, seed=31, kv_len=kv_len, depth=depth, tree=True, nan_tail=True)
    assert all((int(x) - 21) % 16 == 12 for x in kv_len[:4])
    binding.ss_set_option("attn_path", 2)
    try:
        check(inp, oracle, max_q_len=21, label=f"tree depth 20, ctx%16==12, {kv_dtype} {hq}/{hkv}")
    finally:
        binding.ss_set_option("attn_path", 0)
