"""Full-size parity on the 14B-shaped workloads (40/8 heads, D=128, V=151936, bf16), in the launch
configuration the benchmark times: the largest corner of the B x k sweep (B=1024, k=8, about
39 GB of KV) and the ragged dynamic batch (B=1024, k_b in 0..8, per-sequence drafter noise).
The oracle checks a sample of sequences (attention: longest, shortest and a spread; sampler: a
stride through the batch); properties that hold at any size cover the rest."""
import dataclasses

import numpy as np
import pytest
import torch

from helpers import (check_bf16_attention_rows, compare_sampler, flag_bound, gpu_attention, gpu_sample,
                     oracle_attention, oracle_sample)
from paper_2510_26475_amd import synth
from paper_2510_26475_amd.synth import sub_batch

pytestmark = pytest.mark.gpu


def _attention_sample(oracle, batch, seqs):
    out, lse = gpu_attention(batch)
    assert torch.isfinite(out.float()).all() and torch.isfinite(lse).all()
    sb = sub_batch(batch, seqs)
    ref, ref_lse = oracle_attention(oracle, sb)
    qi = batch.q_indptr.tolist()
    rows = torch.tensor([r for b in seqs for r in range(qi[b], qi[b + 1])], device="cuda")
    check_bf16_attention_rows(out[rows].double().cpu().numpy(), ref)
    assert np.abs(lse[rows].double().cpu().numpy() - ref_lse).max() <= 2e-2


def _sampler_sample(oracle, batch, seqs):
    toks, n, flags = gpu_sample(batch, workspace=None)
    k = np.array(batch.k_per_seq)
    # properties at any size: counts within the draft length, accepted tokens are the drafts,
    # one final token, -1 behind it
    assert ((n >= 0) & (n <= k)).all()
    drafts, qi = batch.draft_tokens.cpu().numpy(), batch.q_indptr.cpu().numpy()
    for b in range(len(k)):
        d0 = qi[b] - b
        assert (toks[b, :n[b]] == drafts[d0:d0 + n[b]]).all()
        assert 0 <= toks[b, n[b]] < batch.wl.V and (toks[b, n[b] + 1:] == -1).all()
    sb = sub_batch(batch, seqs)
    ref = oracle_sample(oracle, sb, max_k=batch.max_k)
    tally = compare_sampler((toks[seqs], n[seqs], flags[seqs]), ref)
    assert tally["flagged"] <= flag_bound(len(seqs), batch.wl.V), tally
    return n


def test_sweep_corner_b1024_k8(oracle):
    wl = dataclasses.replace(synth.WORKLOADS["qwen14b_sweep"], B=1024, k=8)
    batch = synth.make_batch(wl, device="cuda", with_logits=False)
    # longest, shortest, and every 32nd sequence
    seqs = sorted(set([int(np.argmax(batch.kv_lens)), int(np.argmin(batch.kv_lens)), 1023] + list(range(0, 1024, 32))))
    _attention_sample(oracle, batch, seqs)
    del batch
    torch.cuda.empty_cache()
    batch = synth.make_batch(wl, device="cuda", with_attention=False)
    n = _sampler_sample(oracle, batch, list(range(0, 1024, 32)))
    assert 1.9 < float((n + 1).mean()) < 3.2          # closed form at sigma = 1, k = 8 is about 2.6


def test_ragged_dynamic_batch_b1024(oracle):
    wl = synth.WORKLOADS["qwen14b_ragged"]
    batch = synth.make_batch(wl, device="cuda", with_logits=False)
    ks = np.array(batch.k_per_seq)
    assert ks.min() == 0 and ks.max() == 8
    pick = [int(np.argmax(batch.kv_lens)), int(np.argmin(batch.kv_lens)), int(np.flatnonzero(ks == 0)[0]),
            int(np.flatnonzero(ks == 8)[0]), int(np.flatnonzero(ks == 3)[0])]
    _attention_sample(oracle, batch, sorted(set(pick + list(range(5, 1024, 32)))))
    del batch
    torch.cuda.empty_cache()
    batch = synth.make_batch(wl, device="cuda", with_attention=False)
    _sampler_sample(oracle, batch, list(range(0, 1024, 32)))
