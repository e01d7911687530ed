"""GPU parity: ss_spec_verify_attn (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

from paper_2604_09562_amd import binding, synth

pytestmark = pytest.mark.gpu

TINY, LLAMA8B, RAGGED, LONG, FP8_70B = synth.CONFIGS


def run_gpu(inp, max_q_len=None, want_lse=True):
    """max_q_len None: the batch's own largest row count, as a caller that runs the depth controller
    passes it; 0: unknown (the library assumes the largest depth it supports)."""
    if max_q_len is None:
        max_q_len = int(np.diff(inp["q_indptr"]).max())
    d = binding.attention_to_device(inp)
    out, lse, ws = binding.alloc_attention_outputs(d, max_q_len=max_q_len)
    ws.fill_(0xFF)  # scratch may hold anything (here NaN patterns)
    out.fill_(0)
    binding.ss_spec_verify_attn(d, out, lse if want_lse else None, ws, max_q_len=max_q_len)
    torch.cuda.synchronize()
    o = out.cpu().numpy().astype(np.float64) if inp["q_dtype"] == "f32" else binding.bf16_bits_to_float(out)
    return o, lse.cpu().numpy().astype(np.float64)


def check(inp, oracle, *, max_q_len=None, requests=None, atol=2e-2, rtol=1e-2, label=""):
    """Tolerance of the benchmark spec: |gpu - ref| <= atol + rtol*|ref| (fp8 caches: atol 6e-2)."""
    if inp["kv_dtype"] == "fp8":
        atol = 6e-2
    ref, ref_lse = oracle.verify_attn(inp, requests=requests)
    got, got_lse = run_gpu(inp, max_q_len)
    sel = ~np.isnan(ref)
    assert sel.any()
    assert np.all(np.isfinite(got[sel])), f"{label}: non-finite output"
    err = np.abs(got - ref)
    bound = atol + rtol * np.abs(ref)
    worst = np.nanmax(np.where(sel, err - bound, -np.inf))
    assert worst <= 0, f"{label}: max abs err {np.nanmax(err[sel]):.4g}, worst excess {worst:.4g}"
    lsel = ~np.isnan(ref_lse)
    assert np.max(np.abs(got_lse[lsel] - ref_lse[lsel])) < 2e-3, f"{label}: lse mismatch"
    return float(np.nanmax(err[sel]))


def test_config0_tiny_fp32(oracle):
    for seed in range(3):
        inp = synth.make_attention_inputs(TINY, seed=seed)
        err = check(inp, oracle, label=f"tiny seed {seed}")
        assert err < 1e-4  # fp32 throughout: far inside the bf16 tolerance


@pytest.mark.parametrize("path", [0, 1])
@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
@pytest.mark.parametrize("hq,hkv", [(8, 8), (8, 4), (16, 4), (16, 2)])
def test_small_shapes_all_groupings(oracle, path, kv_dtype, hq, hkv):
    # several tiles, ragged tails, ragged depths; path 1 forces the fp32 vector kernel
    cfg = LLAMA8B.scaled(batch=6, num_q_heads=hq, num_kv_heads=hkv, kv_dtype=kv_dtype,
                         ctx=("uniform", 9, 700), depth=("uniform", 0, 8))
    inp = synth.make_attention_inputs(cfg, seed=hq + hkv)
    binding.ss_set_option("attn_path", path)
    try:
        check(inp, oracle, label=f"{kv_dtype} {hq}/{hkv} path {path}")
    finally:
        binding.ss_set_option("attn_path", 0)


@pytest.mark.parametrize("max_q_len", [0, 5])
def test_fixed_depth_uses_tight_row_bound(oracle, max_q_len):
    cfg = LLAMA8B.scaled(batch=8, ctx=("uniform", 100, 1500))
    inp = synth.make_attention_inputs(cfg, seed=1)
    check(inp, oracle, max_q_len=max_q_len, label=f"k=4 max_q_len {max_q_len}")


def test_partition_count_invariance(oracle):
    # the same batch with very different numbers of KV partitions must agree with the oracle each time
    cfg = LLAMA8B.scaled(batch=5, ctx=("uniform", 300, 3000), depth=("uniform", 0, 8))
    inp = synth.make_attention_inputs(cfg, seed=2)
    try:
        for waves in (4, 64, 1024, 0):
            binding.ss_set_option("attn_waves", waves)
            check(inp, oracle, label=f"waves {waves}")
    finally:
        binding.ss_set_option("attn_waves", 0)


def test_span_cut_weight_invariance(oracle):
    # where the spans are cut (what opening a unit is charged, in tiles) must not show in the result: many short
    # units, a few long ones, several span counts -- cuts inside units, at unit starts and several units per span
    cfg = LLAMA8B.scaled(batch=24, ctx=("loguniform", 17, 4000), depth=("uniform", 0, 8))
    inp = synth.make_attention_inputs(cfg, seed=11)
    try:
        for weight in (0, 1, 3, 17, 64):
            binding.ss_set_option("attn_unit_weight", weight)
            for waves in (8, 64, 0):
                binding.ss_set_option("attn_waves", waves)
                check(inp, oracle, label=f"unit weight {weight}, waves {waves}")
    finally:
        binding.ss_set_option("attn_unit_weight", 3)
        binding.ss_set_option("attn_waves", 0)


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_repeated_calls_give_the_same_bits(kv_dtype):
    # partials are combined in a fixed order (inside a workgroup and in the merge kernel), so the output may not
    # depend on which wavefront finishes first: eight calls on the full chip, compared bit for bit
    base = LLAMA8B if kv_dtype == "bf16" else FP8_70B
    cfg = base.scaled(batch=48, ctx=("loguniform", 40, 6000), depth=("uniform", 0, 4))
    inp = synth.make_attention_inputs(cfg, seed=13)
    d = binding.attention_to_device(inp)
    mq = int(np.diff(inp["q_indptr"]).max())
    first = None
    for _ in range(8):
        out, lse, ws = binding.alloc_attention_outputs(d, max_q_len=mq)
        ws.fill_(0xFF)
        binding.ss_spec_verify_attn(d, out, lse, ws, max_q_len=mq)
        torch.cuda.synchronize()
        got = (out.view(torch.int16).cpu().numpy().copy(), lse.cpu().numpy().copy())
        if first is None:
            first = got
        else:
            assert np.array_equal(got[0], first[0]) and np.array_equal(got[1], first[1])


def test_edge_lengths(oracle):
    # kv_len equal to q_len (nothing but the new tokens), exact multiples of the block size, one token
    kv_len = np.array([1, 9, 16, 17, 32, 5, 48, 255, 256, 257], np.int32)
    depth = np.array([0, 8, 3, 8, 0, 4, 8, 2, 8, 7], np.int32)
    cfg = LLAMA8B.scaled(batch=len(kv_len))
    inp = synth.make_attention_inputs(cfg, seed=3, kv_len=kv_len, depth=depth)
    check(inp, oracle, label="edge lengths")
    cfg8 = FP8_70B.scaled(batch=len(kv_len))
    inp8 = synth.make_attention_inputs(cfg8, seed=3, kv_len=kv_len, depth=depth)
    check(inp8, oracle, label="edge lengths fp8")


def test_nan_garbage_in_unused_slots(oracle):
    cfg = LLAMA8B.scaled(batch=6, ctx=("uniform", 20, 400), depth=("uniform", 0, 8))
    inp = synth.make_attention_inputs(cfg, seed=4, nan_tail=True)
    check(inp, oracle, label="nan tail bf16")
    cfg8 = FP8_70B.scaled(batch=6, ctx=("uniform", 20, 400))
    inp8 = synth.make_attention_inputs(cfg8, seed=4, nan_tail=True)
    check(inp8, oracle, label="nan tail fp8")


def test_large_scores(oracle):
    cfg = LLAMA8B.scaled(batch=4, ctx=("uniform", 100, 600))
    inp = synth.make_attention_inputs(cfg, seed=5)
    q = synth.decode_storage(inp["q"], "bf16") * 12.0     # scores with std ~12: softmax nearly one-hot
    inp["q"] = synth.to_bf16_bits(q)
    check(inp, oracle, label="large scores")


def test_plan_reuse_across_layers(oracle):
    # Two "layers" of one decode step: the same batch metadata and workspace, different queries and
    # cache contents.  The second call skips the plan kernel and must still match the oracle; with a
    # row bound that needs several passes the flag is ignored and the result is right all the same.
    for cfg, depth in ((LLAMA8B.scaled(batch=9, ctx=("uniform", 30, 2500), depth=("uniform", 0, 8)), None),
                       (FP8_70B.scaled(batch=5, ctx=("uniform", 30, 800)), np.array([20, 3, 11, 0, 16], np.int32))):
        kw = {} if depth is None else dict(depth=depth, kv_len=np.array([300, 41, 800, 17, 129], np.int32))
        layer0 = synth.make_attention_inputs(cfg, seed=8, **kw)
        layer1 = dict(layer0, k_cache=layer0["v_cache"], v_cache=layer0["k_cache"],      # other contents, same layout
                      q=synth.to_bf16_bits(-synth.decode_storage(layer0["q"], "bf16")))
        if cfg.kv_dtype == "fp8":
            layer1.update(k_scale=layer0["v_scale"], v_scale=layer0["k_scale"])
        mq = int(np.diff(layer0["q_indptr"]).max())
        d0, d1 = binding.attention_to_device(layer0), binding.attention_to_device(layer1)
        out, lse, ws = binding.alloc_attention_outputs(d0, max_q_len=mq)
        binding.ss_spec_verify_attn(d0, out, lse, ws, max_q_len=mq)
        for name in ("block_table", "kv_len", "q_indptr"):    # the very same metadata arrays
            d1[name] = d0[name]
        out1 = torch.empty_like(out)
        binding.ss_spec_verify_attn(d1, out1, lse, ws, max_q_len=mq, reuse_plan=True)
        torch.cuda.synchronize()
        ref, _ = oracle.verify_attn(layer1)
        got = binding.bf16_bits_to_float(out1)
        atol = 6e-2 if cfg.kv_dtype == "fp8" else 2e-2
        assert np.all(np.abs(got - ref) <= atol + 1e-2 * np.abs(ref)), cfg.name
        fresh = torch.empty_like(out)
        binding.ss_spec_verify_attn(d1, fresh, lse, ws, max_q_len=mq)
        torch.cuda.synchronize()
        assert torch.equal(fresh, out1), "a reused plan must give the bits a fresh one gives"


def test_empty_batch_is_noop():
    cfg = LLAMA8B.scaled(batch=2, ctx=("fixed", (40,)))
    inp = synth.make_attention_inputs(cfg, seed=0)
    d = binding.attention_to_device(inp)
    out, lse, ws = binding.alloc_attention_outputs(d)
    d0 = dict(d, batch=0, total_rows=0)
    binding.ss_spec_verify_attn(d0, out, lse, ws)
    torch.cuda.synchronize()


def test_argument_errors_are_reported():
    cfg = LLAMA8B.scaled(batch=2, ctx=("fixed", (40,)))
    inp = synth.make_attention_inputs(cfg, seed=0)
    d = binding.attention_to_device(inp)
    out, lse, ws = binding.alloc_attention_outputs(d)
    with pytest.raises(binding.SpecVerifyError, match="workspace"):
        binding.ss_spec_verify_attn(d, out, lse, ws[:256])
    with pytest.raises(binding.SpecVerifyError, match="block_size"):
        binding.ss_spec_verify_attn(dict(d, block_size=32), out, lse, ws)
    with pytest.raises(binding.SpecVerifyError, match="multiple"):
        binding.ss_spec_verify_attn(dict(d, num_q_heads=30), out, lse, ws)
    with pytest.raises(binding.SpecVerifyError, match="scale"):
        binding.ss_spec_verify_attn(dict(d, kv_dtype="fp8"), out, lse, ws)
    torch.cuda.synchronize()


# ---- full-size configurations: the whole batch, element by element, at three seeds ----------------------
FULL = [(LLAMA8B, 5), (RAGGED, 9), (LONG, 7), (FP8_70B, 9)]
FULL_IDS = ["llama3_8b_b64", "ragged_b128", "long_b16", "llama70b_fp8_b96"]


@pytest.mark.timeout(900)
@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("cfg,max_q_len", FULL, ids=FULL_IDS)
def test_full_size_configs_whole_batch(oracle, cfg, max_q_len, seed):
    # the launch configuration the benchmark times (same row bound, automatic partition count); every
    # request, head and row is compared with the oracle
    inp = synth.make_attention_inputs(cfg, seed=seed)
    assert int(np.diff(inp["q_indptr"]).max()) <= max_q_len
    check(inp, oracle, max_q_len=max_q_len, label=f"{cfg.name} seed {seed}")
