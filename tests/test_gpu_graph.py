"""The verify step under HIP graph capture: the library allocates nothing, clears nothing with memsets
and never synchronises, so a captured step must replay to the bits of the eager call, every time."""
import numpy as np
import pytest
import torch

from paper_2604_09562_amd import binding, synth

pytestmark = pytest.mark.gpu

LLAMA8B = synth.CONFIGS[1]


def test_captured_step_replays_exactly():
    cfg = LLAMA8B.scaled(batch=12, vocab=20000, ctx=("uniform", 40, 3000), depth=("uniform", 0, 8))
    att = synth.make_attention_inputs(cfg, seed=5)
    acc = synth.make_accept_inputs(cfg, seed=5, depth=att["depth"])
    mq = int(att["depth"].max()) + 1
    d_att, d_acc = binding.attention_to_device(att), binding.accept_to_device(acc)
    out, lse, ws = binding.alloc_attention_outputs(d_att, max_q_len=mq)
    n_acc, toks, ratio, ws_a = binding.alloc_accept_outputs(d_acc)

    def step():
        binding.ss_spec_verify_attn(d_att, out, lse, ws, max_q_len=mq)
        binding.ss_spec_accept(d_acc, n_acc, toks, ratio, ws_a, max_q_len=mq)

    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in (out, lse, n_acc, toks)]

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for replay in range(4):
        for t in (out, lse, n_acc, toks):
            t.fill_(0)                           # eager work between replays; results must come from the replay
        ws.fill_(0xFF)
        ws_a.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref, name in zip((out, lse, n_acc, toks), want, ("out", "lse", "accepted_len", "out_tokens")):
            assert torch.equal(got, ref), f"replay {replay}: {name} differs from the eager call"
