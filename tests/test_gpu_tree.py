"""GPU parity of the tree-draft entry points against the CPU oracle."""
import math

import numpy as np
import pytest
import torch

from helpers import attn_wgs, env_setting, gpu_attention, gpu_tree_attention, oracle_tree_attention, sub_tree_batch
from paper_2510_26475_amd import binding, synth

pytestmark = pytest.mark.gpu

BF16_TOL, F32_TOL = 2e-2, 1e-5


def _wl(name, Hq, Hkv, D, dtype, V=8):
    return synth.Workload(name, B=0, k=0, Hq=Hq, Hkv=Hkv, D=D, V=V, dtype=dtype,
                          len_dist="uniform", len_lo=1, len_hi=1)


def _check(out, lse, ref, ref_lse, dtype):
    got = out.double().cpu().numpy()
    assert np.isfinite(got).all(), "output holds NaN/inf (a row was not written?)"
    err = np.abs(got - ref)
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    assert err.max() <= tol, f"max abs err {err.max():.3e} > {tol}"
    if dtype == "bf16":
        assert math.sqrt(float((err ** 2).mean())) <= 2.5e-3
    lerr = np.abs(lse.double().cpu().numpy() - ref_lse)
    assert lerr.max() <= (1e-4 if dtype == "f32" else 2e-2)


def _trees(n, seed, max_nodes=12):
    gen = torch.Generator().manual_seed(seed)
    out = []
    for i in range(n):
        kind = i % 4
        if kind == 0:
            out.append(synth.random_parents(1 + int(torch.randint(0, max_nodes, (1,), generator=gen)), gen))
        elif kind == 1:
            out.append(synth.caterpillar_parents(1 + i % 3, 2 + i % 2))
        elif kind == 2:
            out.append(list(range(-1, 1 + i % 5)))      # a chain
        else:
            out.append([-1])                             # no drafts at all
    return out


def test_f32_trees(oracle):
    wl = _wl("tree_f32", 4, 2, 64, "f32")
    pars = _trees(10, 1)
    tb = synth.make_tree_batch(wl, pars, device="cuda", kv_lens=[300, 14, 129, 1, 700, 40, 64, 65, 257, 31],
                               seed=1, with_logits=False)
    out, lse = gpu_tree_attention(tb)
    ref, ref_lse = oracle_tree_attention(oracle, tb)
    _check(out, lse, ref, ref_lse, "f32")


@pytest.mark.parametrize("wgs", [None, 1, 3, 64])
@pytest.mark.parametrize("heads", [(28, 4, 128), (16, 2, 128), (8, 8, 64), (40, 8, 128)])
def test_bf16_trees(oracle, heads, wgs):
    Hq, Hkv, D = heads
    wl = _wl("tree_bf16", Hq, Hkv, D, "bf16")
    pars = _trees(12, 2, max_nodes=8 if Hq // Hkv >= 7 else 12)
    lens = [300, 33, 129, 9, 700, 40, 64, 65, 257, 31, 1025, 96]
    tb = synth.make_tree_batch(wl, pars, device="cuda", kv_lens=lens, seed=2, with_logits=False)
    with attn_wgs(wgs):
        out, lse = gpu_tree_attention(tb)
    ref, ref_lse = oracle_tree_attention(oracle, tb)
    _check(out, lse, ref, ref_lse, "bf16")


def test_chain_mask_equals_the_chain_entry_point_bit_for_bit():
    wl = _wl("tree_chain", 28, 4, 128, "bf16")
    ks = [3, 0, 4, 1, 2, 4]
    lens = [500, 33, 129, 64, 1000, 77]
    tb = synth.make_tree_batch(wl, [list(range(-1, k)) for k in ks], device="cuda", kv_lens=lens, seed=3,
                               with_logits=False)
    out_t, lse_t = gpu_tree_attention(tb)
    batch = synth.VerifyBatch(wl=wl, q=tb.q, k_cache=tb.k_cache, v_cache=tb.v_cache, q_indptr=tb.q_indptr,
                              kv_indptr=tb.kv_indptr, target_logits=torch.empty(0), draft_logits=torch.empty(0),
                              draft_tokens=torch.empty(0), u_accept=torch.empty(0), u_final=torch.empty(0),
                              k_per_seq=ks, kv_lens=lens)
    out_c, lse_c = gpu_attention(batch)
    assert torch.equal(out_t, out_c) and torch.equal(lse_t, lse_c)


@pytest.mark.parametrize("quad", [1, 0])
@pytest.mark.parametrize("wgs", [None, 2, 7])
def test_wide_trees(oracle, wgs, quad):
    # 13 rows x 7 heads per group = 91 columns: one block of 128 columns (quad) or two of 64
    wl = _wl("tree_wide", 28, 4, 128, "bf16")
    pars = [synth.caterpillar_parents(4, 3), synth.caterpillar_parents(3, 4), synth.caterpillar_parents(2, 2),
            synth.caterpillar_parents(6, 2), [-1]]
    tb = synth.make_tree_batch(wl, pars, device="cuda", kv_lens=[600, 200, 90, 1300, 5], seed=4, with_logits=False)
    with env_setting("RESPEC_ATTN_QUAD", quad), attn_wgs(wgs):
        out, lse = gpu_tree_attention(tb)
    ref, ref_lse = oracle_tree_attention(oracle, tb)
    _check(out, lse, ref, ref_lse, "bf16")


def test_headline_tree_workload_sampled_sequences(oracle):
    """B=256, 28/4 heads, a chain of 3 nodes with 2 candidates per position (49 columns) in the
    launch configuration the benchmark times; the oracle checks a sample of sequences."""
    wl = synth.WORKLOADS["qwen7b_b256_k3"]
    tb = synth.make_tree_batch(wl, [synth.caterpillar_parents(3, 2)] * wl.B, device="cuda", with_logits=False)
    out, lse = gpu_tree_attention(tb)
    assert torch.isfinite(out.float()).all()
    seqs = sorted(set([int(np.argmax(tb.kv_lens)), int(np.argmin(tb.kv_lens)), 0, 50, 101, 199, 255]))
    sb = sub_tree_batch(tb, seqs)
    ref, ref_lse = oracle_tree_attention(oracle, sb)
    qi = tb.q_indptr.tolist()
    rows = torch.tensor([r for b in seqs for r in range(qi[b], qi[b + 1])], device="cuda")
    _check(out[rows], lse[rows], ref, ref_lse, "bf16")


def test_more_than_64_rows_is_refused():
    wl = _wl("tree_big", 4, 2, 64, "f32")
    tb = synth.make_tree_batch(wl, [list(range(-1, 63))], device="cuda", kv_lens=[100], seed=5, with_logits=False)
    ws = torch.empty(binding.respec_verify_attention_workspace_bytes(1, 64, 100, 64, 100, 4, 2, 64, 0),
                     dtype=torch.uint8, device="cuda")
    out = torch.empty_like(tb.q)
    with pytest.raises(binding.RespecError) as e:
        binding.respec_verify_attention_tree(tb.q, tb.k_cache, tb.v_cache, tb.q_indptr, tb.kv_indptr,
                                             tb.tree_mask, out, None, 65, 100, 0.125, ws)
    assert e.value.status == 2
