"""GPU parity over several consecutive decode steps: append -> verify attention -> accept -> commit.

The device cache and the host cache each live through all steps (the oracle appends to its own
copy), so a mistake that only shows once state carries over (a stale scale, a wrong length after a
rejection) fails here.  Per step: cache bytes and lengths exact, attention within tolerance, tokens
exact or excused by the oracle's near-tie flag.
"""
import numpy as np
import pytest
import torch

from paper_2604_09562_amd import binding, synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("base_cfg", [synth.CONFIGS[1], synth.CONFIGS[4]], ids=["bf16", "fp8"])
def test_four_steps(oracle, base_cfg):
    cfg = base_cfg.scaled(batch=10, vocab=4096, ctx=("uniform", 150, 420))
    host = synth.make_attention_inputs(cfg, seed=7)          # blocks allocated for the final lengths
    B, Hq, Hkv, D = host["batch"], host["num_q_heads"], host["num_kv_heads"], host["head_dim"]
    cur = host["kv_len"].astype(np.int32) - 40                # valid lengths before the first step
    dev = binding.attention_to_device(host)
    rng = np.random.default_rng(99)
    tol = 6e-2 if cfg.kv_dtype == "fp8" else 2e-2
    for step in range(4):
        depth = rng.integers(0, 9, B).astype(np.int32)
        q_indptr = np.zeros(B + 1, dtype=np.int32)
        q_indptr[1:] = np.cumsum(depth + 1)
        R = int(q_indptr[-1])
        step_in = dict(host, kv_len=(cur + depth + 1).astype(np.int32), depth=depth, q_indptr=q_indptr, total_rows=R,
                       q=synth.store(rng.standard_normal((R, Hq, D), dtype=np.float32), "bf16"),
                       k_new=synth.store(rng.standard_normal((R, Hkv, D), dtype=np.float32), "bf16"),
                       v_new=synth.store(rng.standard_normal((R, Hkv, D), dtype=np.float32), "bf16"), new_dtype="bf16")
        acc_in = synth.make_accept_inputs(cfg, seed=step, depth=depth)

        # device side
        d = dict(dev, depth=depth, total_rows=R, new_dtype="bf16")
        for name in ("kv_len", "q_indptr", "q", "k_new", "v_new"):
            d[name] = binding._to_dev(step_in[name], "cuda:0")
        binding.ss_kv_append(d)
        mq = int(depth.max()) + 1
        out, lse, ws = binding.alloc_attention_outputs(d, max_q_len=mq)
        binding.ss_spec_verify_attn(d, out, lse, ws, max_q_len=mq)
        da = binding.accept_to_device(acc_in)
        n_acc, toks, ratio, ws_a = binding.alloc_accept_outputs(da)
        binding.ss_spec_accept(da, n_acc, toks, ratio, ws_a)
        binding.ss_kv_commit(d["q_indptr"], n_acc, d["kv_len"])
        torch.cuda.synchronize()

        # oracle side (host cache appended in place: step_in shares the cache arrays with `host`)
        oracle.kv_append(step_in)
        ref_out, _ = oracle.verify_attn(step_in)
        ref_acc = oracle.spec_accept(acc_in)

        for name in ("k_cache", "v_cache"):
            assert np.array_equal(dev[name].cpu().numpy().view(np.uint8), host[name].view(np.uint8)), f"step {step}: {name}"
        if cfg.kv_dtype == "fp8":
            used = host["block_table"][host["block_table"] >= 0]
            for name in ("k_scale", "v_scale"):
                assert np.array_equal(dev[name].cpu().numpy()[used], host[name][used]), f"step {step}: {name}"
        got = binding.bf16_bits_to_float(out)
        assert np.all(np.abs(got - ref_out) <= tol + 1e-2 * np.abs(ref_out)), f"step {step}: attention"
        g_n, g_t = n_acc.cpu().numpy(), toks.cpu().numpy()
        n_used = ref_acc["accepted_len"].copy()
        for b in range(B):
            if g_n[b] == ref_acc["accepted_len"][b] and np.array_equal(g_t[b], ref_acc["out_tokens"][b]):
                continue
            first = min(g_n[b], ref_acc["accepted_len"][b])
            d0 = q_indptr[b] - b
            assert g_n[b] != ref_acc["accepted_len"][b] and first < depth[b] and ref_acc["near_tie"][d0 + first] == 1, \
                f"step {step} request {b}: gpu {g_n[b]} {g_t[b].tolist()} oracle {ref_acc['accepted_len'][b]}"
            n_used[b] = g_n[b]   # a near-tie: follow the device's decision so that both sides stay in step
        want_len = oracle.kv_commit(q_indptr, n_used, step_in["kv_len"])
        assert np.array_equal(d["kv_len"].cpu().numpy(), want_len), f"step {step}: lengths after commit"
        cur = want_len


def test_controller_closed_loop(oracle):
    """Depths chosen by the controller from the acceptance each request just saw: the device loop
    (ss_spec_accept + ss_depth_update) and the oracle loop must walk through the same depths."""
    from oracle.depth_controller import DepthController
    cfg = synth.CONFIGS[2].scaled(batch=12, vocab=2048)
    B = cfg.batch
    dev_state = [binding.ss_depth_init() for _ in range(B)]
    ref_state = [DepthController() for _ in range(B)]
    depth_dev = np.full(B, 5, dtype=np.int32)
    depth_ref = depth_dev.copy()
    seen = set()
    for step in range(8):
        assert np.array_equal(depth_dev, depth_ref), f"step {step}: depths diverged"
        acc_in = synth.make_accept_inputs(cfg, seed=step, depth=depth_dev)
        da = binding.accept_to_device(acc_in)
        n_acc, toks, ratio, ws = binding.alloc_accept_outputs(da)
        binding.ss_spec_accept(da, n_acc, toks, ratio, ws)
        torch.cuda.synchronize()
        g_n = n_acc.cpu().numpy()
        ref = oracle.spec_accept(acc_in)
        r_n = ref["accepted_len"].copy()
        for b in range(B):
            if g_n[b] != r_n[b]:    # only a flagged near-tie may differ; then follow the device
                d0 = acc_in["q_indptr"][b] - b
                assert ref["near_tie"][d0 + min(g_n[b], r_n[b])] == 1
                r_n[b] = g_n[b]
        load, tput = 0.2 + 0.05 * step, 150.0 + 60.0 * step
        for b in range(B):
            k = int(depth_dev[b])
            a_dev = g_n[b] / k if k else 0.0
            a_ref = r_n[b] / k if k else 0.0
            depth_dev[b] = binding.ss_depth_update(dev_state[b], a_dev, load, tput)[3]
            depth_ref[b] = ref_state[b].update(a_ref, load, tput)[3]
            seen.add(int(depth_dev[b]))
    assert np.array_equal(depth_dev, depth_ref)
    assert len(seen) > 1, "the controller never moved the depth: the test exercises nothing"
