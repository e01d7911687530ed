"""Option "validate": inconsistent device-resident metadata must come back as an error code, not as a
kernel reading outside its buffers.  The checking kernel itself reads only within the declared sizes, so
these cases are safe to run; with the option off the same valid inputs give the same results."""
import numpy as np
import pytest
import torch

from paper_2604_09562_amd import binding, synth

pytestmark = pytest.mark.gpu

LLAMA8B = synth.CONFIGS[1]


@pytest.fixture()
def validating():
    binding.ss_set_option("validate", 1)
    yield
    binding.ss_set_option("validate", 0)


def attn_case():
    cfg = LLAMA8B.scaled(batch=6, ctx=("uniform", 40, 300), depth=("uniform", 0, 8))
    inp = synth.make_append_inputs(cfg, seed=4)
    return inp


def run_attn(inp):
    d = binding.append_to_device(inp)
    mq = int(inp["depth"].max()) + 1
    out, lse, ws = binding.alloc_attention_outputs(d, max_q_len=mq)
    binding.ss_spec_verify_attn(d, out, lse, ws, max_q_len=mq)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_valid_batch_passes_and_results_do_not_change(validating):
    inp = attn_case()
    with_check = run_attn(inp)
    binding.ss_set_option("validate", 0)
    without = run_attn(inp)
    assert np.array_equal(with_check, without)
    binding.ss_set_option("validate", 1)
    binding.ss_kv_append(binding.append_to_device(inp))
    acc = synth.make_accept_inputs(LLAMA8B.scaled(batch=6, vocab=5000), seed=1)
    da = binding.accept_to_device(acc)
    n, t, r, ws = binding.alloc_accept_outputs(da)
    binding.ss_spec_accept(da, n, t, r, ws)
    torch.cuda.synchronize()


@pytest.mark.parametrize("what", ["block_id_high", "block_id_negative", "kv_len_short", "kv_len_long", "q_len_22",
                                  "q_start", "q_total"])
def test_bad_attention_metadata_is_reported(validating, what):
    inp = attn_case()
    b = 3
    if what == "block_id_high":
        inp["block_table"][b, 1] = inp["num_blocks"] + 5
    elif what == "block_id_negative":
        inp["block_table"][b, 0] = -1
    elif what == "kv_len_short":
        inp["kv_len"][b] = int(inp["depth"][b])          # fewer cache positions than query rows
    elif what == "kv_len_long":
        inp["kv_len"][b] = inp["max_blocks_per_seq"] * 16 + 1
    elif what == "q_len_22":
        inp["q_indptr"][b + 1:] += 22 - (inp["q_indptr"][b + 1] - inp["q_indptr"][b])
        inp["total_rows"] = int(inp["q_indptr"][-1])
        R = inp["total_rows"]
        inp["q"] = np.zeros((R,) + inp["q"].shape[1:], dtype=inp["q"].dtype)
        inp["k_new"] = np.zeros((R,) + inp["k_new"].shape[1:], dtype=inp["k_new"].dtype)
        inp["v_new"] = inp["k_new"].copy()
    elif what == "q_start":
        inp["q_indptr"][0] = 1
    elif what == "q_total":
        inp["q_indptr"][-1] -= 1 if inp["q_indptr"][-1] - inp["q_indptr"][-2] > 1 else -1
    with pytest.raises(binding.SpecVerifyError) as e:
        run_attn(inp)
    msg = str(e.value)
    assert "ss_spec_verify_attn" in msg
    if what.startswith("block_id") or what.startswith("kv_len"):
        assert f"request {b}" in msg
    with pytest.raises(binding.SpecVerifyError):
        binding.ss_kv_append(binding.append_to_device(inp))


def test_row_bound_hint_smaller_than_the_batch_needs(validating):
    inp = attn_case()
    d = binding.append_to_device(inp)
    mq = int(inp["depth"].max())          # one less than the longest request has rows
    out, lse, ws = binding.alloc_attention_outputs(d, max_q_len=mq)
    with pytest.raises(binding.SpecVerifyError) as e:
        binding.ss_spec_verify_attn(d, out, lse, ws, max_q_len=mq)
    assert "query rows" in str(e.value)


@pytest.mark.parametrize("what", ["token", "temperature", "uniform"])
def test_bad_accept_inputs_are_reported(validating, what):
    acc = synth.make_accept_inputs(LLAMA8B.scaled(batch=6, vocab=5000), seed=2)
    if what == "token":
        acc["draft_tokens"][7] = 5000
    elif what == "temperature":
        acc["temperature"][2] = 0.0
    else:
        acc["u_sample"][4] = 1.0
    da = binding.accept_to_device(acc)
    n, t, r, ws = binding.alloc_accept_outputs(da)
    with pytest.raises(binding.SpecVerifyError):
        binding.ss_spec_accept(da, n, t, r, ws)
