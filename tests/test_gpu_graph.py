"""The verify step under HIP graph capture: the library allocates nothing, never synchronises
and records no memset, so attention + sampling can be captured once and replayed.  Every replay
(with eager work between the replays) must reproduce the eager results bit for bit."""
import math

import pytest
import torch

from paper_2510_26475_amd import binding, synth

pytestmark = pytest.mark.gpu


def test_verify_step_replays_from_a_graph():
    wl = synth.Workload("graph", B=24, k=3, Hq=28, Hkv=4, D=128, V=151936, dtype="bf16",
                        len_dist="uniform", len_lo=100, len_hi=3000, seed=21)
    dev = torch.device("cuda:0")
    batch = synth.make_batch(wl, device=dev)
    B, max_q = wl.B, batch.max_k + 1
    ws = torch.empty(binding.respec_verify_attention_workspace_bytes(
        B, batch.total_q, batch.total_kv, max_q, batch.max_kv_len, wl.Hq, wl.Hkv, wl.D, binding.RESPEC_BF16),
        dtype=torch.uint8, device=dev)
    out = torch.empty_like(batch.q)
    lse = torch.empty((batch.total_q, wl.Hq), dtype=torch.float32, device=dev)
    toks = torch.empty((B, batch.max_k + 1), dtype=torch.int32, device=dev)
    n_acc = torch.empty((B,), dtype=torch.int32, device=dev)
    flags = torch.empty((B,), dtype=torch.int32, device=dev)

    def step():
        binding.respec_verify_attention(batch.q, batch.k_cache, batch.v_cache, batch.q_indptr, batch.kv_indptr,
                                        out, lse, max_q, batch.max_kv_len, 1.0 / math.sqrt(wl.D), ws)
        binding.respec_rejection_sample(batch.target_logits, batch.draft_logits, batch.draft_tokens,
                                        batch.q_indptr, batch.u_accept, batch.u_final, toks, n_acc, flags,
                                        batch.max_k, wl.temperature)

    step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (out, lse, toks, n_acc, flags)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()
    for _ in range(4):
        for t in (out, lse, toks, n_acc, flags):
            t.zero_()                            # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (out, lse, toks, n_acc, flags)
        assert torch.equal(got[0].view(torch.int16), ref[0].view(torch.int16))
        assert all(torch.equal(a, b) for a, b in zip(got[1:], ref[1:]))
