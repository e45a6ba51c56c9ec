"""GPU parity of the paged-cache entry points against the CPU oracle: attention through a page
table (chain and tree masks) and the in-place commit of accepted tokens."""
import math

import numpy as np
import pytest
import torch

from helpers import (attn_wgs, gpu_attention, gpu_paged_attention, gpu_tree_attention, gpu_tree_sample,
                     oracle_paged_attention, oracle_tree_sample)
from paper_2510_26475_amd import binding, synth

pytestmark = pytest.mark.gpu

BF16_TOL, F32_TOL = 2e-2, 1e-5


def _wl(name, Hq, Hkv, D, dtype, V=8):
    return synth.Workload(name, B=0, k=0, Hq=Hq, Hkv=Hkv, D=D, V=V, dtype=dtype,
                          len_dist="uniform", len_lo=1, len_hi=1)


def _check(out, lse, ref, ref_lse, dtype):
    got = out.double().cpu().numpy()
    assert np.isfinite(got).all(), "output holds NaN/inf (an unused slot was read, or a row was not written)"
    err = np.abs(got - ref)
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    assert err.max() <= tol, f"max abs err {err.max():.3e} > {tol}"
    if dtype == "bf16":
        assert math.sqrt(float((err ** 2).mean())) <= 2.5e-3
    lerr = np.abs(lse.double().cpu().numpy() - ref_lse)
    assert lerr.max() <= (1e-4 if dtype == "f32" else 2e-2)


LENS = [33, 130, 257, 1000, 6, 5, 128, 129, 2049, 16, 17, 48]
KS = [3, 4, 0, 4, 4, 4, 1, 2, 3, 0, 4, 2]


@pytest.mark.parametrize("page_size", [16, 32, 64])
def test_f32_chain_and_tree(oracle, page_size):
    wl = _wl("paged_f32", 4, 2, 64, "f32")
    batch = synth.make_batch(wl, device="cuda", kv_lens=LENS, k_per_seq=KS, seed=1, with_logits=False)
    pk = synth.paginate(batch.k_cache, batch.v_cache, batch.kv_lens, page_size, seed=page_size, extra_pages_per_seq=1)
    out, lse = gpu_paged_attention(batch, pk)
    ref, ref_lse = oracle_paged_attention(oracle, batch, pk)
    _check(out, lse, ref, ref_lse, "f32")
    parents = [synth.caterpillar_parents(2, 2), [-1, 0, 0, 1, 1, 2], [-1], list(range(-1, 4))]
    tb = synth.make_tree_batch(wl, parents, device="cuda", kv_lens=[300, 14, 129, 40], seed=2, with_logits=False)
    pk = synth.paginate(tb.k_cache, tb.v_cache, tb.kv_lens, page_size, seed=3)
    out, lse = gpu_paged_attention(tb, pk, tree_mask=tb.tree_mask)
    ref, ref_lse = oracle_paged_attention(oracle, tb, pk, tree_mask=tb.tree_mask)
    _check(out, lse, ref, ref_lse, "f32")


@pytest.mark.parametrize("wgs", [None, 1, 3, 64])
@pytest.mark.parametrize("page_size", [16, 32, 64, 256])
@pytest.mark.parametrize("heads", [(28, 4, 128), (16, 2, 128), (8, 2, 64)])
def test_bf16_paged_equals_oracle_and_the_contiguous_entry_point(oracle, heads, page_size, wgs):
    Hq, Hkv, D = heads
    wl = _wl("paged_bf16", Hq, Hkv, D, "bf16")
    batch = synth.make_batch(wl, device="cuda", kv_lens=LENS, k_per_seq=KS, seed=Hq + page_size, with_logits=False)
    pk = synth.paginate(batch.k_cache, batch.v_cache, batch.kv_lens, page_size, seed=page_size + (wgs or 0),
                        spare_pages=7)
    with attn_wgs(wgs):
        out, lse = gpu_paged_attention(batch, pk)
        flat_out, flat_lse = gpu_attention(batch)
    ref, ref_lse = oracle_paged_attention(oracle, batch, pk)
    _check(out, lse, ref, ref_lse, "bf16")
    # the same tiles in the same order: the page table must not change a single bit
    assert torch.equal(out, flat_out) and torch.equal(lse, flat_lse)


@pytest.mark.parametrize("page_size", [16, 64])
def test_bf16_paged_tree_with_wide_column_blocks(oracle, page_size):
    wl = _wl("paged_tree", 28, 4, 128, "bf16")
    parents = [synth.caterpillar_parents(3, 2), synth.caterpillar_parents(2, 3), [-1], [-1, 0, 0, 1, 1, 2],
               synth.caterpillar_parents(4, 2)]
    tb = synth.make_tree_batch(wl, parents, device="cuda", kv_lens=[700, 33, 129, 9, 2050], seed=5, with_logits=False)
    pk = synth.paginate(tb.k_cache, tb.v_cache, tb.kv_lens, page_size, seed=6, extra_pages_per_seq=2)
    out, lse = gpu_paged_attention(tb, pk, tree_mask=tb.tree_mask)
    ref, ref_lse = oracle_paged_attention(oracle, tb, pk, tree_mask=tb.tree_mask)
    _check(out, lse, ref, ref_lse, "bf16")
    flat_out, flat_lse = gpu_tree_attention(tb)
    assert torch.equal(out, flat_out) and torch.equal(lse, flat_lse)


def test_headline_workload_paged_sampled_sequences(oracle):
    """B=256, k=3, 28/4 heads at full size through 16-token pages; sampled sequences against the
    oracle, every element against the contiguous entry point."""
    wl = synth.WORKLOADS["qwen7b_b256_k3"]
    batch = synth.make_batch(wl, device="cuda", with_logits=False)
    pk = synth.paginate(batch.k_cache, batch.v_cache, batch.kv_lens, 16, seed=1, spare_pages=100)
    out, lse = gpu_paged_attention(batch, pk)
    flat_out, flat_lse = gpu_attention(batch)
    assert torch.equal(out, flat_out) and torch.equal(lse, flat_lse)
    # (the contiguous entry point's own full-size test checks sampled sequences against the oracle)


def _bits(t):
    return t.view(torch.int16 if t.element_size() == 2 else torch.int32)


# (8 KV heads in fp32: a token is 4096 B = 256 sixteen-byte pieces, so every wave of the commit
# kernel's work-group moves data and every wave's view of the old length matters)
@pytest.mark.parametrize("dtype,Hkv", [("f32", 4), ("bf16", 4), ("f32", 8)])
@pytest.mark.parametrize("page_size", [16, 64])
def test_commit_matches_the_oracle_bit_for_bit(oracle, dtype, Hkv, page_size):
    wl = _wl("commit", 2 * Hkv, Hkv, 128, dtype)
    parents = [synth.caterpillar_parents(3, 3), [-1, 0, 0, 2, 2, 4], [-1, 0], synth.caterpillar_parents(2, 2),
               synth.caterpillar_parents(3, 3), [-1], list(range(-1, 5))]
    lens = [50, 8, 2, 21, 33, 70, 19]
    tb = synth.make_tree_batch(wl, parents, device="cuda", kv_lens=lens, seed=7, with_logits=False)
    pk = synth.paginate(tb.k_cache, tb.v_cache, tb.kv_lens, page_size, seed=8, extra_pages_per_seq=1)
    path = torch.tensor([[1, 4, 9, -1, -1], [2, 4, 5, -1, -1], [-1] * 5, [1, -1, -1, -1, -1], [3, -1, -1, -1, -1],
                         [-1] * 5, [1, 2, 3, 4, 5]], dtype=torch.int32, device="cuda")
    n = torch.tensor([3, 3, 0, 1, 1, 0, 5], dtype=torch.int32, device="cuda")
    odt = oracle.F32 if dtype == "f32" else oracle.BF16
    kp, vp = synth.to_host_array(pk.k_pages).copy(), synth.to_host_array(pk.v_pages).copy()
    kv_len = pk.kv_len.cpu().numpy().copy()
    oracle.commit_accepted_paged(kp, vp, tb.q_indptr.cpu().numpy(), pk.page_indptr.cpu().numpy(),
                                 pk.page_table.cpu().numpy(), kv_len, n.cpu().numpy(), odt, path=path.cpu().numpy())
    binding.respec_commit_accepted_paged(pk.k_pages, pk.v_pages, tb.q_indptr, pk.page_indptr, pk.page_table,
                                         pk.kv_len, n, tb.total_q, tb.max_rows, path=path)
    torch.cuda.synchronize()
    assert pk.kv_len.cpu().tolist() == kv_len.tolist()
    host = (lambda a: a.view(np.int32)) if dtype == "f32" else (lambda a: a.view(np.int16))
    np.testing.assert_array_equal(_bits(pk.k_pages).cpu().numpy(), host(kp))
    np.testing.assert_array_equal(_bits(pk.v_pages).cpu().numpy(), host(vp))


def test_chain_commit_only_cuts_the_length():
    wl = _wl("commit_chain", 8, 4, 128, "bf16")
    ks = [4, 3, 0, 2]
    batch = synth.make_batch(wl, device="cuda", kv_lens=[30, 9, 5, 17], k_per_seq=ks, seed=9, with_logits=False)
    pk = synth.paginate(batch.k_cache, batch.v_cache, batch.kv_lens, 16, seed=10)
    k0, v0 = _bits(pk.k_pages).clone(), _bits(pk.v_pages).clone()
    n = torch.tensor([2, 3, 0, 0], dtype=torch.int32, device="cuda")
    binding.respec_commit_accepted_paged(pk.k_pages, pk.v_pages, batch.q_indptr, pk.page_indptr, pk.page_table,
                                         pk.kv_len, n, batch.total_q, 5)
    torch.cuda.synchronize()
    assert torch.equal(_bits(pk.k_pages), k0) and torch.equal(_bits(pk.v_pages), v0)
    assert pk.kv_len.cpu().tolist() == [30 - 4 + 2, 9 - 3 + 3, 5, 17 - 2]


def test_verify_commit_then_plain_decode(oracle):
    """A speculative step followed by a non-speculative one on the same cache: tree verify,
    sampling, commit, then one decode row (k = 0) per sequence over the committed cache; the
    oracle does the same on its own copy."""
    wl = synth.Workload("transition", B=0, k=0, Hq=16, Hkv=2, D=128, V=4096, dtype="bf16",
                        len_dist="uniform", len_lo=1, len_hi=1, sigma=1.0)
    parents = [synth.caterpillar_parents(3, 2)] * 6 + [[-1]] * 2 + [synth.caterpillar_parents(2, 3)] * 4
    lens = [200, 37, 64, 65, 1000, 16, 300, 5, 129, 48, 23, 512]
    tb = synth.make_tree_batch(wl, parents, device="cuda", kv_lens=lens, seed=11)
    pk = synth.paginate(tb.k_cache, tb.v_cache, tb.kv_lens, 16, seed=12, extra_pages_per_seq=1, poison=True)
    B = len(parents)
    # GPU: sample, commit
    g_tok, g_path, g_n, g_flags = gpu_tree_sample(tb)
    r_tok, r_path, r_n, r_flags = oracle_tree_sample(oracle, tb)
    keep = r_flags == 0
    assert (g_n[keep] == r_n[keep]).all() and (g_path[keep] == r_path[keep]).all()
    # commit what the ORACLE accepted on both sides, so that a flagged draw cannot make the caches differ
    n_dev = torch.tensor(r_n, dtype=torch.int32, device="cuda")
    path_dev = torch.tensor(r_path, dtype=torch.int32, device="cuda")
    kp, vp = synth.to_host_array(pk.k_pages).copy(), synth.to_host_array(pk.v_pages).copy()
    kv_len = pk.kv_len.cpu().numpy().copy()
    oracle.commit_accepted_paged(kp, vp, tb.q_indptr.cpu().numpy(), pk.page_indptr.cpu().numpy(),
                                 pk.page_table.cpu().numpy(), kv_len, r_n, oracle.BF16, path=r_path)
    binding.respec_commit_accepted_paged(pk.k_pages, pk.v_pages, tb.q_indptr, pk.page_indptr, pk.page_table,
                                         pk.kv_len, n_dev, tb.total_q, tb.max_rows, path=path_dev)
    torch.cuda.synchronize()
    assert pk.kv_len.cpu().tolist() == kv_len.tolist()
    # the next step: the K/V of the token drawn last is appended at position kv_len, then one
    # decode row per sequence attends over the whole committed cache
    gen = torch.Generator(device="cuda").manual_seed(13)
    q = torch.randn((B, wl.Hq, wl.D), generator=gen, device="cuda").to(torch.bfloat16)
    new_k = torch.randn((B, wl.Hkv, wl.D), generator=gen, device="cuda").to(torch.bfloat16)
    new_v = torch.randn((B, wl.Hkv, wl.D), generator=gen, device="cuda").to(torch.bfloat16)
    ps = pk.page_size
    e = pk.page_indptr[:-1].long() + (pk.kv_len.long() // ps)
    slot = pk.page_table[e].long() * ps + pk.kv_len.long() % ps
    pk.k_pages.view(-1, wl.Hkv, wl.D)[slot] = new_k
    pk.v_pages.view(-1, wl.Hkv, wl.D)[slot] = new_v
    pk.kv_len += 1
    slot_h = slot.cpu().numpy()
    kp.reshape(-1, wl.Hkv, wl.D)[slot_h] = synth.to_host_array(new_k)
    vp.reshape(-1, wl.Hkv, wl.D)[slot_h] = synth.to_host_array(new_v)
    kv_len += 1
    dec = synth.VerifyBatch(wl=wl, q=q, k_cache=torch.empty(0), v_cache=torch.empty(0),
                            q_indptr=torch.arange(B + 1, dtype=torch.int32, device="cuda"), kv_indptr=torch.empty(0),
                            target_logits=torch.empty(0), draft_logits=torch.empty(0), draft_tokens=torch.empty(0),
                            u_accept=torch.empty(0), u_final=torch.empty(0), k_per_seq=[0] * B, kv_lens=kv_len.tolist())
    out, lse = gpu_paged_attention(dec, pk, max_rows=1)
    ref, ref_lse = oracle.verify_attention_paged(
        synth.to_host_array(q), kp, vp, np.arange(B + 1, dtype=np.int32), pk.page_indptr.cpu().numpy(),
        pk.page_table.cpu().numpy(), kv_len, wl.Hq, wl.Hkv, wl.D, float(np.float32(1.0 / math.sqrt(wl.D))),
        oracle.BF16, want_lse=True, n_threads=0)
    _check(out, lse, ref, ref_lse, "bf16")


def test_next_layer_on_a_paged_cache_is_bit_equal_to_a_full_call(oracle):
    """Another layer's K/V pools behind the same page table: the set-up in the workspace is reused."""
    wl = _wl("paged_layers", 28, 4, 128, "bf16")
    batch = synth.make_batch(wl, device="cuda", kv_lens=LENS, k_per_seq=KS, seed=41, with_logits=False)
    pk = synth.paginate(batch.k_cache, batch.v_cache, batch.kv_lens, 16, seed=42, extra_pages_per_seq=1)
    g = torch.Generator(device="cuda").manual_seed(43)
    k2 = torch.empty_like(pk.k_pages).normal_(generator=g)      # layer 2: other values in the same slots
    v2 = torch.empty_like(pk.v_pages).normal_(generator=g)
    q2 = torch.empty_like(batch.q).normal_(generator=g)
    B, max_rows, max_kv = pk.kv_len.numel(), max(KS) + 1, int(pk.kv_len.max())
    ws = torch.empty(binding.respec_verify_attention_workspace_bytes(
        B, batch.total_q, pk.num_pages * pk.page_size, max_rows, max_kv, wl.Hq, wl.Hkv, wl.D, binding.RESPEC_BF16),
        dtype=torch.uint8, device="cuda")

    def run(entry, q, kp, vp):
        out = torch.full_like(q, float("nan"))
        lse = torch.full((batch.total_q, wl.Hq), float("nan"), dtype=torch.float32, device="cuda")
        entry(q, kp, vp, batch.q_indptr, pk.page_indptr, pk.page_table, pk.kv_len, out, lse, max_rows, max_kv,
              1.0 / math.sqrt(wl.D), ws)
        torch.cuda.synchronize()
        return out, lse

    full2 = run(binding.respec_verify_attention_paged, q2, k2, v2)
    ws.zero_()
    run(binding.respec_verify_attention_paged, batch.q, pk.k_pages, pk.v_pages)              # layer 1 sets up
    next2 = run(binding.respec_verify_attention_paged_next_layer, q2, k2, v2)               # layer 2 reuses
    assert torch.equal(full2[0].view(torch.int16), next2[0].view(torch.int16)) and torch.equal(full2[1], next2[1])
    ref, ref_lse = oracle.verify_attention_paged(
        synth.to_host_array(q2), synth.to_host_array(k2), synth.to_host_array(v2), batch.q_indptr.cpu().numpy(),
        pk.page_indptr.cpu().numpy(), pk.page_table.cpu().numpy(), pk.kv_len.cpu().numpy(), wl.Hq, wl.Hkv, wl.D,
        float(np.float32(1.0 / math.sqrt(wl.D))), oracle.BF16, tree_mask=None, want_lse=True, n_threads=0)
    _check(next2[0], next2[1], ref, ref_lse, "bf16")


def test_bad_arguments_are_rejected_before_any_launch():
    wl = _wl("paged_err", 4, 2, 64, "f32")
    batch = synth.make_batch(wl, device="cuda", kv_lens=[40, 20], k_per_seq=[1, 1], seed=1, with_logits=False)
    for ps, status in ((8, 2), (24, 2), (2048, 2)):
        pk = synth.paginate(batch.k_cache, batch.v_cache, batch.kv_lens, ps, seed=0)
        with pytest.raises(binding.RespecError) as e:
            gpu_paged_attention(batch, pk)
        assert e.value.status == status
        n = torch.zeros(2, dtype=torch.int32, device="cuda")
        with pytest.raises(binding.RespecError) as e:
            binding.respec_commit_accepted_paged(pk.k_pages, pk.v_pages, batch.q_indptr, pk.page_indptr,
                                                 pk.page_table, pk.kv_len, n, batch.total_q, 2)
        assert e.value.status == status
