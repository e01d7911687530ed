#!/usr/bin/env python3
"""Benchmark of the verify step (spec_verify_attn + spec_accept) on one MI355X.

One "step" = one pass of the whole hot path over one synthetic batch: the KV
plan, the KV-streaming attention kernel, the partial merge, and the five accept
passes.  Inputs are resident in HBM before the timed region; several copies of
the cache and logits are rotated so the last-level cache cannot serve the stream.
Prints ONE JSON line: metric, value (verified tokens/s), roofline of the KV-streaming kernel, CPU-oracle baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


ATTN_SOURCES = ("attn_mfma_kernels.h", "attn_mfma.hip", "common.h", "tree_window.h", "span_cuts.h")


def attn_source_hash() -> str:
    """Hash of the sources the streaming kernel is built from (ties a counter measurement to a kernel version)."""
    import hashlib
    h = hashlib.sha256()
    for name in ATTN_SOURCES:
        with open(os.path.join(ROOT, "paper_2604_09562_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str):
    """HBM bytes per launch of the streaming kernel from the committed counter summary, with its provenance.

    The figure comes from two rocprofv3 --pmc runs of this script (FETCH_SIZE, WRITE_SIZE) scaled by the
    calibration copy; the summary file carries it on a line `traffic_bytes_per_launch: N` and the hash of the
    kernel sources it was measured on (`kernel_source_hash: H`).  A summary taken on other sources is not
    reported as this kernel's traffic: the value is None and the reason is in the second return value."""
    rel = os.path.join("profiles", f"attn_stream_kernel_{workload}_hbm_traffic.txt")
    val = tag = None
    try:
        with open(os.path.join(ROOT, rel)) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    val = float(line.split(":", 1)[1])
                if line.startswith("kernel_source_hash:"):
                    tag = line.split(":", 1)[1].strip()
    except OSError:
        return None, "no counter summary for this workload"
    now = attn_source_hash()
    if val is None:
        return None, f"{rel} holds no traffic line"
    if tag != now:
        return None, f"{rel} was measured on kernel sources {tag}, these are {now}"
    return val, f"{rel} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, kernel sources {now})"


def cpu_baseline(cfg, att, acc, budget_requests: int):
    """The oracle as it stands, timed on this host on the first `budget_requests` requests."""
    import oracle
    n = min(budget_requests, att["batch"])
    reqs = list(range(n))
    sub = dict(acc)
    rows = int(acc["q_indptr"][n])
    sub.update(batch=n, total_rows=rows, q_indptr=acc["q_indptr"][:n + 1], depth=acc["depth"][:n],
               target_logits=acc["target_logits"][:rows], draft_logits=acc["draft_logits"][:max(rows - n, 0)],
               draft_tokens=acc["draft_tokens"][:rows - n], u_accept=acc["u_accept"][:rows - n],
               u_sample=acc["u_sample"][:n], temperature=acc["temperature"][:n])
    # whole passes over the sample until about ten seconds of wall time have gone by
    t_att = t_acc = 0.0
    passes = 0
    while passes < 200 and t_att + t_acc < 10.0:
        t0 = time.perf_counter()
        oracle.verify_attn(att, requests=reqs)
        t1 = time.perf_counter()
        oracle.spec_accept(sub)
        t2 = time.perf_counter()
        t_att += t1 - t0
        t_acc += t2 - t1
        passes += 1
    toks = rows
    return dict(value=passes * toks / (t_att + t_acc), unit="verified tokens/s", cores=oracle.num_threads(), kind="oracle",
                sample=f"first {n} of {att['batch']} requests ({toks} query tokens), {passes} passes in "
                       f"{t_att + t_acc:.1f} s: attention {t_att / passes:.3f} s, accept {t_acc / passes:.3f} s per pass")


def cpu_baseline_one_thread(att, acc, n: int = 4):
    """The same oracle on one host thread, on the first `n` requests, one pass."""
    import oracle
    n = min(n, att["batch"])
    rows = int(acc["q_indptr"][n])
    sub = dict(acc)
    sub.update(batch=n, total_rows=rows, q_indptr=acc["q_indptr"][:n + 1], depth=acc["depth"][:n],
               target_logits=acc["target_logits"][:rows], draft_logits=acc["draft_logits"][:max(rows - n, 0)],
               draft_tokens=acc["draft_tokens"][:rows - n], u_accept=acc["u_accept"][:rows - n],
               u_sample=acc["u_sample"][:n], temperature=acc["temperature"][:n])
    t0 = time.perf_counter()
    oracle.verify_attn(att, requests=list(range(n)), threads=1)
    t1 = time.perf_counter()
    oracle.spec_accept(sub, threads=1)
    t2 = time.perf_counter()
    return dict(value=rows / (t2 - t0), unit="verified tokens/s", cores=1, kind="oracle",
                sample=f"first {n} of {att['batch']} requests ({rows} query tokens), one pass: attention {t1 - t0:.3f} s, "
                       f"accept {t2 - t1:.3f} s")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="llama3_8b_b64")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--rotate", type=int, default=4, help="distinct copies of cache and logits cycled through")
    ap.add_argument("--cpu-requests", type=int, default=-1,
                    help="requests in the CPU-oracle sample (0 = skip, -1 = the whole batch)")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="after timing, launch a plain device copy of this size three times: the known-size "
                         "kernel that scales FETCH_SIZE / WRITE_SIZE in a rocprofv3 --pmc run of this command")
    ap.add_argument("--no-check", action="store_true", help="skip the parity spot check after timing")
    ap.add_argument("--graph", action="store_true",
                    help="replay each step from a captured HIP graph (the kernel durations of the roofline entry "
                         "then come from an eager pass after the timed region)")
    ap.add_argument("--depth", type=int, default=-1,
                    help="give every request this draft depth instead of the workload's own (0..20; for what-if runs)")
    ap.add_argument("--tree", action="store_true",
                    help="the drafts of every request form a random tree instead of a chain (same shapes and sizes)")
    ap.add_argument("--attn-waves", type=int, default=0, help="KV partitions of the attention kernel (0 = automatic)")
    ap.add_argument("--repeats", type=int, default=5,
                    help="timed regions of --steps steps each; ms_per_step is their median, the spread is reported")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the verify step of one decode lane); "
              "--gpus must be 1", file=sys.stderr)
        return 2

    import torch
    from paper_2604_09562_amd import binding, synth

    if not os.path.exists(binding.LIB_PATH):
        from paper_2604_09562_amd import build
        build.build()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU fallback", file=sys.stderr)
        return 3
    cfg = synth.config_by_name(args.config)
    if args.depth >= 0:
        cfg = cfg.scaled(name=f"{cfg.name}_k{args.depth}", depth=("fixed", args.depth))
    if args.attn_waves:
        binding.ss_set_option("attn_waves", args.attn_waves)
    dev = "cuda:0"
    torch.cuda.set_device(0)

    att = synth.make_attention_inputs(cfg, seed=args.seed, tree=args.tree)
    acc = synth.make_accept_inputs(cfg, seed=args.seed, depth=att["depth"])
    max_q_len = int(att["depth"].max()) + 1
    kv_bytes = synth.kv_bytes_algorithmic(att)
    q_tokens = int(att["total_rows"])

    # device copies (rotated), outputs and workspaces allocated once
    nrot = max(1, args.rotate)
    d_att = [binding.attention_to_device(att, dev) for _ in range(nrot)]
    d_acc = [binding.accept_to_device(acc, dev) for _ in range(nrot)]
    out, lse, ws_att = binding.alloc_attention_outputs(d_att[0], dev, max_q_len=max_q_len)
    n_acc, toks, ratio, ws_acc = binding.alloc_accept_outputs(d_acc[0], dev)

    def step(i: int) -> None:
        binding.ss_spec_verify_attn(d_att[i % nrot], out, lse, ws_att, max_q_len=max_q_len)
        binding.ss_spec_accept(d_acc[i % nrot], n_acc, toks, None, ws_acc, max_q_len=max_q_len)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if args.graph:
        # one graph per rotated copy, captured on a side stream; the timed loop only replays
        graphs, side = [], torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for r in range(nrot):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=side):
                    step(r)
                graphs.append(g)
        torch.cuda.current_stream().wait_stream(side)
        for r in range(nrot):
            graphs[r].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[(args.warmup + i) % nrot].replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        binding.ss_profile_begin(args.steps)
        for i in range(args.steps):
            step(args.warmup + i)
        torch.cuda.synchronize()
    else:
        binding.ss_profile_begin(args.steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    kern_ms = binding.ss_profile_collect(args.steps)
    # The same region again (no kernel events this time): one region is a few milliseconds, so its clock
    # carries a few per cent of noise; the line reports the median region and the spread.
    regions = [1e3 * (t1 - t0) / args.steps]
    for r in range(1, max(1, args.repeats)):
        torch.cuda.synchronize()
        ta = time.perf_counter()
        for i in range(args.steps):
            if args.graph:
                graphs[(args.warmup + i) % nrot].replay()
            else:
                step(args.warmup + i)
        torch.cuda.synchronize()
        regions.append(1e3 * (time.perf_counter() - ta) / args.steps)
    ms_per_step = float(np.median(regions))
    elapsed = ms_per_step * 1e-3 * args.steps

    # per-call breakdown (outside the timed region)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    t_att, t_acc, t_greedy = [], [], []
    for i in range(10):
        ev[0].record()
        binding.ss_spec_verify_attn(d_att[i % nrot], out, lse, ws_att, max_q_len=max_q_len)
        ev[1].record()
        binding.ss_spec_accept(d_acc[i % nrot], n_acc, toks, None, ws_acc, max_q_len=max_q_len)
        ev[2].record()
        torch.cuda.synchronize()
        t_att.append(ev[0].elapsed_time(ev[1]))
        t_acc.append(ev[1].elapsed_time(ev[2]))
    t_reuse = []
    for i in range(10):   # a later layer of the same step: the workspace's plan is still valid
        ev[0].record()
        binding.ss_spec_verify_attn(d_att[i % nrot], out, lse, ws_att, max_q_len=max_q_len, reuse_plan=True)
        ev[1].record()
        torch.cuda.synchronize()
        t_reuse.append(ev[0].elapsed_time(ev[1]))
    accepted = n_acc.cpu().numpy()
    g_acc, g_toks = torch.empty_like(n_acc), torch.empty_like(toks)
    for i in range(6):
        ev[0].record()
        binding.ss_spec_accept(d_acc[i % nrot], g_acc, g_toks, None, ws_acc, greedy=True, max_q_len=max_q_len)
        ev[1].record()
        torch.cuda.synchronize()
        t_greedy.append(ev[0].elapsed_time(ev[1]))

    kern_avg_ms = float(np.mean(kern_ms)) if len(kern_ms) else float("nan")
    achieved = kv_bytes / (kern_avg_ms * 1e-3) / 1e9
    esz = 2 if cfg.logit_dtype == "bf16" else 4
    accept_bytes = (2 * q_tokens - att["batch"]) * cfg.vocab * esz
    traffic, traffic_source = measured_traffic(cfg.name)
    step_bytes = kv_bytes + accept_bytes
    result = {
        "metric": "verified tokens/s + KV read GB/s (% HBM peak), spec_verify_attn+accept, 1 GPU",
        "value": q_tokens * args.steps / elapsed,
        "unit": "verified tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "timed_regions": len(regions), "ms_per_step_min": float(np.min(regions)), "ms_per_step_max": float(np.max(regions)),
        "step_algorithmic_bytes": step_bytes, "step_frac": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"bf16": "bf16", "fp8": "fp8_e4m3", "f32": "f32"}[cfg.kv_dtype], "data": "synthetic",
        "config": {"workload": cfg.name, "batch": att["batch"], "num_q_heads": cfg.num_q_heads,
                   "num_kv_heads": cfg.num_kv_heads, "head_dim": cfg.head_dim, "query_tokens": q_tokens,
                   "kv_tokens": int(att["kv_len"].astype(np.int64).sum()), "vocab": cfg.vocab,
                   "max_q_len": max_q_len, "rotated_copies": nrot, "seed": args.seed,
                   "drafts": "tree" if args.tree else "chain",
                   "launch": "graph replay" if args.graph else "eager",
                   "step": "plan + attention + merge + accept; the plan is rebuilt in every step (t_attn_reused_plan_ms: "
                           "a later layer of the same decode step, which reuses it)"},
        "roofline": {"bound": "hbm", "kernel": "attn_stream_kernel", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes": kv_bytes, "kernel_ms_avg": kern_avg_ms,
                     "kernel_ms_min": float(np.min(kern_ms)) if len(kern_ms) else None, "launches": int(len(kern_ms))},
        "kv_read_gbps": achieved, "pct_hbm_peak": 100.0 * achieved / HBM_PEAK_GBPS,
        "t_attn_ms": float(np.median(t_att)), "t_attn_reused_plan_ms": float(np.median(t_reuse)),
        "t_accept_ms": float(np.median(t_acc)),
        "t_accept_greedy_ms": float(np.median(t_greedy)),
        "accept_pass1_gbps": accept_bytes / (float(np.median(t_acc)) * 1e-3) / 1e9,
        "emitted_tokens_per_s": float((accepted + 1).sum()) * args.steps / elapsed,
        "mean_accepted_len": float(accepted.mean()),
    }
    if not args.no_check:
        # spot check after timing: the timed path must still agree with the oracle on one request
        import oracle
        b = int(np.argmax(att["kv_len"]))
        ref, _ = oracle.verify_attn(att, requests=[b])
        got = binding.bf16_bits_to_float(out) if cfg.q_dtype != "f32" else out.cpu().numpy().astype(np.float64)
        r0, r1 = att["q_indptr"][b], att["q_indptr"][b + 1]
        err = float(np.max(np.abs(got[r0:r1] - ref[r0:r1])))
        result["spot_check_max_abs_err"] = err
        tol = 6e-2 if cfg.kv_dtype == "fp8" else 2e-2
        if not err <= tol + 1e-2 * float(np.max(np.abs(ref[r0:r1]))):
            print(f"bench.py: parity spot check failed (max abs err {err})", file=sys.stderr)
            return 4
    if not args.no_check:
        # acceptance of the whole batch against the oracle, with the near-tie accounting the method's statement asks for:
        # a request may differ only from a draft on whose ratio test the uniform lies within 1e-5 of min(1, p/q)
        import oracle
        binding.ss_spec_accept(d_acc[0], n_acc, toks, None, ws_acc, max_q_len=max_q_len)
        torch.cuda.synchronize()
        ref = oracle.spec_accept(acc)
        g_n, g_t = n_acc.cpu().numpy(), toks.cpu().numpy()
        excused, wrong = 0, []
        for b in range(att["batch"]):
            if g_n[b] == ref["accepted_len"][b] and np.array_equal(g_t[b], ref["out_tokens"][b]):
                continue
            first, d0 = int(min(g_n[b], ref["accepted_len"][b])), int(acc["q_indptr"][b]) - b
            if (g_n[b] != ref["accepted_len"][b] and first < acc["depth"][b] and ref["near_tie"][d0 + first] == 1
                    and np.array_equal(g_t[b, :first], ref["out_tokens"][b, :first])):
                excused += 1
            else:
                wrong.append(b)
        result["near_tie_flagged"] = int(ref["near_tie"].sum())       # drafts with |u - min(1, p/q)| < 1e-5 (oracle)
        result["near_tie_excused"] = excused                           # requests that differ, starting at such a draft
        result["cdf_tie_range_mean"] = float(np.mean(ref["y_hi"] - ref["y_lo"] + 1))   # tokens within 1e-5 of u_sample's CDF point
        result["accept_requests_equal"] = int(att["batch"] - excused - len(wrong))
        if wrong:
            print(f"bench.py: acceptance differs from the oracle in requests {wrong[:8]}", file=sys.stderr)
            return 4
    # the steps around the verify step (not part of the timed step): append the new tokens' K/V, commit lengths
    rng = np.random.default_rng(args.seed)
    shape = (q_tokens, cfg.num_kv_heads, cfg.head_dim)
    new_dtype = "f32" if cfg.kv_dtype == "f32" else "bf16"
    d_app = dict(d_att[0], new_dtype=new_dtype,
                 k_new=binding._to_dev(synth.store(rng.standard_normal(shape, dtype=np.float32), new_dtype), dev),
                 v_new=binding._to_dev(synth.store(rng.standard_normal(shape, dtype=np.float32), new_dtype), dev))
    lens = d_att[0]["kv_len"].clone()
    t_app, t_com = [], []
    for i in range(8):
        ev[0].record()
        binding.ss_kv_append(d_app, max_q_len=max_q_len)
        ev[1].record()
        binding.ss_kv_commit(d_att[0]["q_indptr"], n_acc, lens)
        ev[2].record()
        torch.cuda.synchronize()
        t_app.append(ev[0].elapsed_time(ev[1]))
        t_com.append(ev[1].elapsed_time(ev[2]))
        lens.copy_(d_att[0]["kv_len"])
    if args.tree:
        # the acceptance calls for tree-shaped drafts on the same trees (outside the timed step, which runs the chain rule)
        tr = synth.make_tree_sample_inputs(cfg, seed=args.seed, depth=att["depth"])
        d_tr = binding.accept_to_device(tr, dev)
        nodes = torch.empty((att["batch"], binding.SS_MAX_DEPTH), dtype=torch.int32, device=dev)
        ws_tr = binding.tree_sample_workspace(d_tr, dev)
        t_tg, t_ts = [], []
        for i in range(6):
            ev[0].record()
            binding.ss_spec_accept_tree_greedy(d_tr, g_acc, g_toks, nodes, ws_acc, max_q_len=max_q_len)
            ev[1].record()
            binding.ss_spec_accept_tree_sample(d_tr, g_acc, g_toks, nodes, None, ws_tr, max_q_len=max_q_len)
            ev[2].record()
            torch.cuda.synchronize()
            t_tg.append(ev[0].elapsed_time(ev[1]))
            t_ts.append(ev[1].elapsed_time(ev[2]))
        result["t_tree_accept_greedy_ms"] = float(np.median(t_tg))
        result["t_tree_accept_sample_ms"] = float(np.median(t_ts))
    result["t_kv_append_ms"] = float(np.median(t_app))
    result["t_kv_commit_ms"] = float(np.median(t_com))
    if args.cpu_requests != 0:
        n_cpu = att["batch"] if args.cpu_requests < 0 else args.cpu_requests
        result["cpu_baseline"] = cpu_baseline(cfg, att, acc, n_cpu)
        result["cpu_baseline_one_thread"] = cpu_baseline_one_thread(att, acc)
    if args.calibrate_copy > 0:
        src = torch.empty(args.calibrate_copy << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
