"""Seeded sweep over small random shapes: every combination the fixed cases may have missed (grouping,
cache dtype, chain or tree, row bound given or not, depths up to 20, lengths around block boundaries),
attention, accept, append and compaction against the oracle."""
import numpy as np
import pytest
import torch

from paper_2604_09562_amd import binding, synth
from tests.test_gpu_attn import check
from tests.test_gpu_accept import compare as compare_accept
from tests.test_gpu_kv import run_and_compare as append_and_compare
from tests.test_gpu_tree_sample import compare as compare_tree_sample
from tests.test_oracle_kv_compact import random_paths

pytestmark = pytest.mark.gpu

LLAMA8B, FP8_70B = synth.CONFIGS[1], synth.CONFIGS[4]


def draw_case(rng):
    hq, hkv = [(8, 8), (8, 4), (16, 4), (16, 2), (32, 8), (64, 8)][int(rng.integers(6))]
    base = FP8_70B if rng.random() < 0.4 else LLAMA8B
    batch = int(rng.integers(1, 12))
    kmax = int(rng.choice([0, 3, 8, 8, 12, 20]))
    depth = rng.integers(0, kmax + 1, batch).astype(np.int32)
    # lengths: some barely above the new tokens, some around block multiples, some long
    kv_len = np.array([int(rng.choice([d + 1, d + 1 + rng.integers(0, 40), 16 * rng.integers(1, 30) + rng.integers(-1, 2),
                                       rng.integers(200, 3000)])) for d in depth], np.int32)
    kv_len = np.maximum(kv_len, depth + 1)
    cfg = base.scaled(batch=batch, num_q_heads=hq, num_kv_heads=hkv, vocab=int(rng.choice([1000, 4096, 20011])))
    return cfg, kv_len, depth, bool(rng.random() < 0.5), bool(rng.random() < 0.7)


@pytest.mark.parametrize("case", range(64))
def test_random_shape(oracle, case):
    rng = np.random.default_rng(1000 + case)
    cfg, kv_len, depth, tree, hinted = draw_case(rng)
    label = f"case {case}: {cfg.kv_dtype} {cfg.num_q_heads}/{cfg.num_kv_heads} B={cfg.batch} depths {depth.tolist()} tree={tree} hint={hinted}"
    print(label, flush=True)
    mq = int(depth.max()) + 1 if hinted else 0

    app = synth.make_append_inputs(cfg, seed=case, kv_len=kv_len, depth=depth, tree=tree)
    append_and_compare(app, oracle, label + " append")          # leaves the appended cache in `app`
    check(app, oracle, max_q_len=mq, label=label + " attention")

    pad = (-cfg.vocab) % 8
    if tree:
        acc = synth.make_tree_accept_inputs(cfg, seed=case, depth=depth, hit=0.75, row_pad=pad)
        ref = oracle.tree_accept_greedy(acc)
        da = binding.accept_to_device({**acc, "draft_logits": None, "u_accept": None, "u_sample": None, "temperature": None})
        n_acc, toks, _, ws = binding.alloc_accept_outputs(da)
        nodes = torch.full((cfg.batch, binding.SS_MAX_DEPTH), -77, dtype=torch.int32, device="cuda:0")
        binding.ss_spec_accept_tree_greedy(da, n_acc, toks, nodes, ws, max_q_len=mq)
        torch.cuda.synchronize()
        assert np.array_equal(n_acc.cpu().numpy(), ref["accepted_len"]), label
        assert np.array_equal(toks.cpu().numpy(), ref["out_tokens"]), label
        assert np.array_equal(nodes.cpu().numpy(), ref["accepted_nodes"]), label
        if case % 2:   # the sampled walk over the same trees
            compare_tree_sample(synth.make_tree_sample_inputs(cfg, seed=case, depth=depth, row_pad=pad), oracle,
                                label + " sampled walk", max_q_len=mq)
        # compaction of a random root path (deeper than the greedy walk usually gets)
        path_nodes, path_len = random_paths(app, case)
        d = binding.attention_to_device(app)
        binding.ss_kv_compact(d, binding.to_device(path_nodes, "cuda:0"), binding.to_device(path_len, "cuda:0"), max_q_len=mq)
        torch.cuda.synchronize()
        oracle.kv_compact(app, path_nodes, path_len)
        for name in ("k_cache", "v_cache"):
            assert np.array_equal(d[name].cpu().numpy().view(np.uint8), app[name].view(np.uint8)), label + " " + name
    else:
        greedy = bool(rng.random() < 0.3)
        acc = synth.make_accept_inputs(cfg, seed=case, depth=depth, greedy=greedy, row_pad=pad)
        compare_accept(acc, oracle, greedy=greedy, label=label + " accept")
