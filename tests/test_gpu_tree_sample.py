"""GPU parity of ss_spec_accept_tree_sample against the CPU oracle.

Token ids, lengths and paths must be exact.  As for the chain rule, the one excused difference is a
node whose uniform lies within 1e-5 of min(1, r/q): the oracle flags those; a request whose first
disagreement is on a flagged node is counted and not compared further.
"""
import numpy as np
import pytest
import torch

from paper_2604_09562_amd import binding, synth

pytestmark = pytest.mark.gpu

TINY, LLAMA8B, RAGGED, LONG, FP8_70B = synth.CONFIGS


def run_gpu(inp, max_q_len=0):
    d = binding.accept_to_device(inp)
    acc, toks, ratio, _ = binding.alloc_accept_outputs(d)
    nodes = torch.full((inp["batch"], binding.SS_MAX_DEPTH), -77, dtype=torch.int32, device="cuda:0")
    ws = binding.tree_sample_workspace(d)
    ws.fill_(0xFF)
    binding.ss_spec_accept_tree_sample(d, acc, toks, nodes, ratio, ws, max_q_len=max_q_len)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), toks.cpu().numpy(), nodes.cpu().numpy(), ratio.cpu().numpy()


def first_disagreement(k, gpu_nodes, gpu_ratio, ref_nodes, ref_ratio):
    """Lowest-numbered node (1..k) whose treatment differs: offered by one side only, or accepted by one side only.

    Nodes are offered in increasing node order (children follow their parent, later siblings follow a
    rejected one), so the lowest differing node is the first decision the two walks do not share.
    `*_ratio[i-1]` is NaN for a node that was never offered.  Returns 0 if every decision agrees."""
    g_acc, r_acc = set(int(x) for x in gpu_nodes if x > 0), set(int(x) for x in ref_nodes if x > 0)
    for i in range(1, k + 1):
        g_off, r_off = not np.isnan(gpu_ratio[i - 1]), not np.isnan(ref_ratio[i - 1])
        if g_off != r_off or ((i in g_acc) != (i in r_acc)):
            return i
    return 0


def compare(inp, oracle, label, max_q_len=0):
    ref = oracle.tree_accept_sample(inp)
    acc, toks, nodes, ratio = run_gpu(inp, max_q_len)
    excused, drafts = 0, 0
    excused_req = set()
    for b in range(inp["batch"]):
        d0, k = inp["q_indptr"][b] - b, int(inp["depth"][b])
        drafts += k
        same = (acc[b] == ref["accepted_len"][b] and np.array_equal(toks[b], ref["out_tokens"][b])
                and np.array_equal(nodes[b], ref["accepted_nodes"][b]))
        if same:
            continue
        # excused only if the first decision the two walks do not share is the accept/reject of a node that both
        # offered and that the oracle flagged as a near-tie; a differing draw after identical decisions never is
        i = first_disagreement(k, nodes[b], ratio[d0:d0 + k], ref["accepted_nodes"][b], ref["ratio"][d0:d0 + k])
        ok = (i > 0 and not np.isnan(ratio[d0 + i - 1]) and not np.isnan(ref["ratio"][d0 + i - 1])
              and ref["near_tie"][d0 + i - 1] == 1)
        assert ok, (
            f"{label}: request {b}: first differing node {i}: gpu n={acc[b]} tokens={toks[b].tolist()} nodes={nodes[b].tolist()} "
            f"oracle n={ref['accepted_len'][b]} tokens={ref['out_tokens'][b].tolist()} nodes={ref['accepted_nodes'][b].tolist()}")
        excused += 1
        excused_req.add(b)
    # with p/q known to about 2e-6 relative, an excusal needs u within that of the ratio: a once-in-1e5 event per draft
    assert excused <= max(1, int(1e-4 * drafts)), f"{label}: {excused} near-tie excusals among {drafts} drafts"
    Rd = inp["total_rows"] - inp["batch"]
    if Rd:
        r = ref["ratio"]
        keep = np.ones(Rd, bool)
        for b in excused_req:   # past an excused request's first difference the walks offer different nodes
            keep[inp["q_indptr"][b] - b:inp["q_indptr"][b + 1] - b - 1] = False
        assert np.array_equal(np.isnan(r[keep]), np.isnan(ratio[:Rd][keep])), f"{label}: different nodes were offered"
        both = keep & np.isfinite(r) & (r < 1e6) & np.isfinite(ratio[:Rd])
        assert np.allclose(ratio[:Rd][both], r[both], rtol=2e-5, atol=1e-30), f"{label}: ratios differ"
    print(f"[tree sample parity] {label}: {inp['batch']} requests, excused {excused}, flagged nodes {int(ref['near_tie'].sum())}, "
          f"mean accepted {acc.mean():.2f}, offered nodes {int(np.isfinite(ref['ratio']).sum())} of {Rd}")
    return ref


@pytest.mark.parametrize("logit_dtype", ["f32", "bf16"])
def test_small_and_odd_vocabularies(oracle, logit_dtype):
    for vocab in (1000, 8192, 20011, 50257):
        pad = (-vocab) % (8 if logit_dtype == "bf16" else 4)
        cfg = TINY.scaled(batch=10, vocab=vocab, logit_dtype=logit_dtype, depth=("uniform", 0, 8), sigma_draft=("fixed", 0.6))
        compare(synth.make_tree_sample_inputs(cfg, seed=vocab % 5, row_pad=pad), oracle, f"vocab {vocab} {logit_dtype}")


def test_full_vocabulary_batches(oracle):
    ref = compare(synth.make_tree_sample_inputs(RAGGED.scaled(batch=32), seed=1), oracle, "ragged trees, 128k vocabulary")
    assert ref["accepted_len"].max() >= 2 and ref["accepted_len"].min() == 0
    compare(synth.make_tree_sample_inputs(LLAMA8B.scaled(batch=16, depth=("uniform", 0, 8)), seed=2), oracle,
            "spiked targets", max_q_len=9)


def test_chain_parents_give_the_chain_result(oracle):
    cfg = LLAMA8B.scaled(batch=24, vocab=20000, depth=("uniform", 0, 8), sigma_draft=("fixed", 0.5))
    inp = synth.make_accept_inputs(cfg, seed=3)
    inp["tree_parent"] = np.concatenate([np.arange(-1, k) for k in inp["depth"]]).astype(np.int32)
    acc, toks, nodes, _ = run_gpu(inp)
    chain = oracle.spec_accept(inp)
    for b in range(24):
        if acc[b] == chain["accepted_len"][b] and np.array_equal(toks[b], chain["out_tokens"][b]):
            continue
        # only a different accepted length whose first differing draft the oracle flagged as a near-tie is excused
        first, d0 = min(acc[b], chain["accepted_len"][b]), inp["q_indptr"][b] - b
        assert (acc[b] != chain["accepted_len"][b] and first < inp["depth"][b] and chain["near_tie"][d0 + first] == 1
                and np.array_equal(toks[b, :first], chain["out_tokens"][b, :first])), f"request {b}"
    compare(inp, oracle, "chain as tree")


def test_depth_20_and_degenerate_proposals(oracle):
    cfg = LLAMA8B.scaled(batch=6, vocab=4096, sigma_draft=("fixed", 0.3))
    depth = np.array([20, 0, 13, 20, 1, 9], np.int32)
    inp = synth.make_tree_sample_inputs(cfg, seed=4, depth=depth)
    compare(inp, oracle, "deep trees")
    # proposal equal to the target row: every offered child is accepted (ratio 1), nothing is ever rejected
    same = synth.make_tree_sample_inputs(cfg, seed=5, depth=depth)
    V = 4096
    for b in range(6):
        r0 = int(same["q_indptr"][b])
        for i in range(1, int(depth[b]) + 1):
            same["draft_logits"][r0 - b + i - 1, :V] = same["target_logits"][r0 + int(same["tree_parent"][r0 + i]), :V]
    ref = compare(same, oracle, "proposal == target")
    tested = np.isfinite(ref["ratio"])
    assert np.allclose(ref["ratio"][tested], 1.0, rtol=1e-9)


def test_argument_errors():
    cfg = TINY.scaled(batch=2, depth=("fixed", 2))
    inp = synth.make_tree_sample_inputs(cfg, seed=0)
    d = binding.accept_to_device(inp)
    acc, toks, ratio, ws_small = binding.alloc_accept_outputs(d)
    nodes = torch.zeros((2, binding.SS_MAX_DEPTH), dtype=torch.int32, device="cuda:0")
    with pytest.raises(binding.SpecVerifyError, match="workspace"):
        binding.ss_spec_accept_tree_sample(d, acc, toks, nodes, ratio, ws_small)   # the chain workspace is too small
    ws = binding.tree_sample_workspace(d)
    with pytest.raises(binding.SpecVerifyError):
        binding.ss_spec_accept_tree_sample({**d, "u_sample": None}, acc, toks, nodes, ratio, ws)
