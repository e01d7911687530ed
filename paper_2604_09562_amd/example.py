"""A decode lane driven end to end through the library, on synthetic model outputs.

    python -m paper_2604_09562_amd.example [--steps N] [--batch B] [--layers L] [--tree]

Each step does what a decode worker does around its model (whose projections and logits are stood in
for by seeded random tensors, there being no weights here):

  router      pick the worker for a new request from reported metrics         ss_route_select
  controller  per request, the next draft depth from its last acceptance     ss_depth_update
  append      write the k+1 new tokens' keys/values into the paged cache      ss_kv_append
  attention   verify attention, once per layer; layers after the first        ss_spec_verify_attn
              reuse the first one's plan                                      (SS_BATCH_REUSE_PLAN)
  accept      acceptance walk and the draw of the next token                  ss_spec_accept, or for draft trees
                                                                              ss_spec_accept_tree_greedy / _sample + ss_kv_compact
  commit      new valid lengths                                               ss_kv_commit

and prints the accepted tokens per step.  Every device step runs in the library's kernels; this file
only moves arguments.
"""
from __future__ import annotations

import argparse
import time

import numpy as np
import torch

from . import binding, synth


def run(steps: int = 6, batch: int = 8, layers: int = 4, tree: bool = False, vocab: int = 32000, seed: int = 0,
        verbose: bool = True, sample: bool = False) -> dict:
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = synth.CONFIGS[1].scaled(batch=batch, vocab=vocab, ctx=("uniform", 200, 1500))
    rng = np.random.default_rng(seed)

    # the router places a new request on one of four workers (host arithmetic)
    # (cache hit rate, memory utilisation, queue depth, active load, stale) as each worker reports them
    workers = [(float(rng.uniform(0, 1)), float(rng.uniform(0.2, 0.9)), int(rng.integers(0, 40)), float(rng.uniform(0, 1)), 0)
               for _ in range(4)]
    chosen = binding.ss_route_select(workers, q_max=64.0)

    # a paged cache with room for every step's tokens; `cur` = valid lengths before the step
    room = steps * (binding.SS_MAX_DEPTH + 1)
    host = synth.make_attention_inputs(cfg, seed=seed)
    cur = np.maximum(host["kv_len"].astype(np.int32) - room, 1)
    cache = binding.attention_to_device(host, dev)
    Hq, Hkv, D = cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim
    ctrl = [binding.ss_depth_init() for _ in range(batch)]
    depth = np.full(batch, 4, dtype=np.int32)
    emitted, t_dev = 0, 0.0
    start_len = cur.copy()

    for step in range(steps):
        # ---- what the models would hand over: draft tokens/logits, queries and new keys/values per layer
        if tree and sample:
            acc = synth.make_tree_sample_inputs(cfg, seed=seed + step, depth=depth)
        elif tree:
            acc = synth.make_tree_accept_inputs(cfg, seed=seed + step, depth=depth, hit=0.7)
        else:
            acc = synth.make_accept_inputs(cfg, seed=seed + step, depth=depth)
        q_indptr, R = acc["q_indptr"], acc["total_rows"]
        mq = int(depth.max()) + 1
        d = dict(cache, depth=depth, total_rows=R, new_dtype="bf16")
        d["kv_len"] = binding.to_device((cur + depth + 1).astype(np.int32), dev)
        d["q_indptr"] = binding.to_device(q_indptr, dev)
        if tree:
            d["tree_mask"] = binding.to_device(acc["tree_mask"], dev)
        for name, heads in (("q", Hq), ("k_new", Hkv), ("v_new", Hkv)):
            d[name] = binding.to_device(synth.store(rng.standard_normal((R, heads, D), dtype=np.float32), "bf16"), dev)
        da = binding.accept_to_device(acc, dev)
        out, lse, ws = binding.alloc_attention_outputs(d, dev, max_q_len=mq)
        n_acc, toks, _, ws_a = binding.alloc_accept_outputs(da, dev)
        nodes = torch.empty((batch, binding.SS_MAX_DEPTH), dtype=torch.int32, device=dev)
        ws_t = binding.tree_sample_workspace(da, dev) if tree and sample else None

        # ---- the device side of the step
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        binding.ss_kv_append(d, max_q_len=mq)
        for layer in range(layers):   # one cache stands in for every layer's; the batch metadata is shared
            binding.ss_spec_verify_attn(d, out, lse, ws, max_q_len=mq, reuse_plan=layer > 0)
        if tree:
            if sample:
                binding.ss_spec_accept_tree_sample(da, n_acc, toks, nodes, None, ws_t, max_q_len=mq)
            else:
                binding.ss_spec_accept_tree_greedy(da, n_acc, toks, nodes, ws_a, max_q_len=mq)
            binding.ss_kv_compact(d, nodes, n_acc, max_q_len=mq)
        else:
            binding.ss_spec_accept(da, n_acc, toks, None, ws_a, max_q_len=mq)
        binding.ss_kv_commit(d["q_indptr"], n_acc, d["kv_len"])
        torch.cuda.synchronize()
        t_dev += time.perf_counter() - t0

        # ---- feedback: the controller turns each request's acceptance into its next depth
        n = n_acc.cpu().numpy()
        cur = d["kv_len"].cpu().numpy()
        load, tput = 0.3, 300.0
        for b in range(batch):
            a = n[b] / depth[b] if depth[b] else 0.0
            depth[b] = binding.ss_depth_update(ctrl[b], float(a), load, tput)[3]
        emitted += int(n.sum()) + batch
        if verbose:
            print(f"step {step}: accepted {n.tolist()} -> next depths {depth.tolist()}")
    if verbose:
        print(f"router chose worker {chosen}; {emitted} tokens emitted in {steps} steps, "
              f"{1e3 * t_dev / steps:.3f} ms of device work per step ({layers} layers)")
    return dict(chosen=chosen, emitted=emitted, depths=depth.copy(), kv_len=cur, start_len=start_len)


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--steps", type=int, default=6)
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--layers", type=int, default=4)
    ap.add_argument("--tree", action="store_true", help="tree-shaped drafts (greedy acceptance unless --sample)")
    ap.add_argument("--sample", action="store_true", help="with --tree: the sampled acceptance walk")
    a = ap.parse_args()
    run(a.steps, a.batch, a.layers, a.tree, sample=a.sample)


if __name__ == "__main__":
    main()
