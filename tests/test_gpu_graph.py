"""The decode step's entry points only enqueue kernels on the caller's stream (no allocation,
no synchronisation, no memset), so a caller can capture them into a HIP graph: a captured step
(attention + log-probs) replayed several times, with eager work and synchronisations between the
replays and changed inputs, must give the eager results bit for bit every time."""
import numpy as np
import pytest
import torch

from paper_2602_09578_amd import binding as B
from paper_2602_09578_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,pdiv,ldiv", [("tiny", 1, 1), ("qwen7b", 32, 8)])
def test_captured_step_replays_bit_identical(name, pdiv, ldiv):
    print("case: graph", name, flush=True)
    w = I.WORKLOADS[name].scaled(pdiv, ldiv) if pdiv > 1 else I.WORKLOADS[name]
    dev = I.build_attn_inputs(w, device="cuda")
    lp = I.build_logprob_inputs(w.num_seqs, min(w.vocab, 32768), w.logit_sigma, w.seed).to("cuda")
    call = B.prepare_attn(dev, B.MARL_OUT_BF16)
    lp_out = torch.empty(w.num_seqs, dtype=torch.float32, device="cuda")
    lp_ws = B.alloc_workspace(B.marl_logprobs_workspace_bytes(*lp.logits.shape), "cuda")

    def step():
        B.run_attn(dev, call)
        B.marl_token_logprobs(lp.logits, lp.tokens, lp.temperature, lp_out, lp_ws)

    step()                                   # warm-up: the library's one-time device queries happen here
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()

    gen = torch.Generator(device="cuda").manual_seed(3)
    for rep in range(4):
        # new queries, lengths and logits in place (the graph holds the addresses, not the contents)
        dev.q.copy_(torch.randn(dev.q.shape, generator=gen, device="cuda").to(torch.bfloat16))
        if rep % 2 == 1:
            dev.suffix_lens.copy_(torch.clamp(dev.suffix_lens - 1, min=0))
        lp.logits.copy_((torch.randn(lp.logits.shape, generator=gen, device="cuda") * 2).to(torch.bfloat16))
        torch.cuda.synchronize()
        step()                               # eager
        torch.cuda.synchronize()
        want_attn, want_lp = call.out.clone(), lp_out.clone()
        call.out.zero_(); lp_out.zero_()
        _ = (dev.q.float() ** 2).sum().item()    # unrelated eager work and a synchronisation in between
        graph.replay()
        torch.cuda.synchronize()
        assert B.marl_attn_read_flags(call.workspace) == 0
        assert torch.equal(call.out.view(torch.int16), want_attn.view(torch.int16)), rep
        assert torch.equal(lp_out.view(torch.int32), want_lp.view(torch.int32)), rep
