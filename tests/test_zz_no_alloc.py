"""ss_spec_accept_static (no workspace, no allocation) against ss_spec_accept on the same inputs.

Two calls in a row through the C ABI, the second on a smaller batch: the static scratch then still holds the first
call's partial results, which must not leak into the second.  Outputs have to equal the workspace entry point's
bit for bit (the two share their kernels); the oracle comparison of those outputs is in test_gpu_accept.py.
"""
import numpy as np
import pytest
import torch

from paper_2604_09562_amd import binding, synth

pytestmark = pytest.mark.gpu

TINY, LLAMA8B, RAGGED, LONG, FP8_70B = synth.CONFIGS


def _both(inp, greedy=False):
    d = binding.accept_to_device(inp)
    mq = int(inp["depth"].max()) + 1
    acc0, toks0, ratio0, ws = binding.alloc_accept_outputs(d)
    binding.ss_spec_accept(d, acc0, toks0, ratio0, ws, greedy=greedy, max_q_len=mq)
    acc1, toks1, ratio1, _ = binding.alloc_accept_outputs(d)
    binding.ss_spec_accept_static(d, acc1, toks1, ratio1, greedy=greedy, max_q_len=mq)
    torch.cuda.synchronize()
    return (acc0.cpu().numpy(), toks0.cpu().numpy(), ratio0.cpu().numpy()), (acc1.cpu().numpy(), toks1.cpu().numpy(), ratio1.cpu().numpy())


def _same(a, b, label):
    assert np.array_equal(a[0], b[0]), f"{label}: accepted lengths differ"
    assert np.array_equal(a[1], b[1]), f"{label}: tokens differ"
    assert np.array_equal(a[2], b[2], equal_nan=True), f"{label}: ratios differ"


def test_two_calls_in_a_row_second_one_smaller(oracle):
    big = synth.make_accept_inputs(RAGGED.scaled(batch=48), seed=5)                      # 128k vocabulary, depths 0..8
    small = synth.make_accept_inputs(RAGGED.scaled(batch=7, vocab=20011), seed=6, row_pad=(-20011) % 8)
    assert binding.lib().ss_spec_accept_workspace(big["batch"], big["total_rows"], big["vocab"]) <= binding.ss_spec_accept_static_capacity()
    a0, a1 = _both(big)
    _same(a0, a1, "first call")
    b0, b1 = _both(small)
    _same(b0, b1, "second, smaller call")
    g0, g1 = _both(small, greedy=True)
    _same(g0, g1, "greedy call")
    # and the results are the method's: the oracle agrees on the second call (no near-tie in this seed)
    ref = oracle.spec_accept(small)
    assert np.array_equal(b1[0], ref["accepted_len"]) and np.array_equal(b1[1], ref["out_tokens"])


def test_sizes_beyond_the_static_buffer_are_rejected():
    cfg = RAGGED.scaled(batch=512, vocab=152064)
    cap = binding.ss_spec_accept_static_capacity()
    need = binding.lib().ss_spec_accept_workspace(512, 512 * 9, 152064)
    assert need > cap
    one = torch.zeros(16, dtype=torch.int32, device="cuda:0")
    d = dict(batch=512, vocab=152064, row_stride=152064, logit_dtype="bf16", total_rows=512 * 9, greedy=0,
             q_indptr=one, target_logits=one, draft_logits=one, draft_tokens=one, u_accept=one, u_sample=one,
             temperature=one)
    with pytest.raises(binding.SpecVerifyError, match="static buffer"):
        binding.ss_spec_accept_static(d, one, one, None)   # rejected on the host: nothing is launched, no pointer is read
    torch.cuda.synchronize()
    del cfg
