"""Pins of the oracle's paged-cache functions (CPU only): attention over a page table and the
commit of accepted tokens.  The reference side of every check is written here with numpy
indexing of its own, or is a property that holds whatever the layout."""
import math

import numpy as np
import pytest
import torch

from paper_2510_26475_amd import synth


def _wl(Hq, Hkv, D, dtype="f32"):
    return synth.Workload("paged", B=0, k=0, Hq=Hq, Hkv=Hkv, D=D, V=8, dtype=dtype,
                          len_dist="uniform", len_lo=1, len_hi=1)


def _dense(q, k, v, G, scale, visible):
    """q [R,Hq,D], k/v [L,Hkv,D] float64, visible [R,L] bool -> out [R,Hq,D] by plain numpy."""
    kq = np.repeat(k, G, axis=1)
    vq = np.repeat(v, G, axis=1)
    s = scale * np.einsum("rhd,lhd->rhl", q, kq)
    s = np.where(visible[:, None, :], s, -np.inf)
    p = np.exp(s - s.max(axis=-1, keepdims=True))
    p /= p.sum(axis=-1, keepdims=True)
    return np.einsum("rhl,lhd->rhd", p, vq)


def _gathered(pk: synth.PagedKV, b):
    """Sequence b's K and V in token order, by this test's own indexing."""
    ps = pk.page_size
    table = pk.page_table.numpy()[int(pk.page_indptr[b]):int(pk.page_indptr[b + 1])]
    L = int(pk.kv_len[b])
    k = np.concatenate([pk.k_pages.numpy()[p] for p in table], axis=0)[:L]
    v = np.concatenate([pk.v_pages.numpy()[p] for p in table], axis=0)[:L]
    assert k.shape[0] == L and ps * len(table) >= L
    return k.astype(np.float64), v.astype(np.float64)


def _chain_visible(R, L):
    i = np.arange(R)[:, None]
    return np.arange(L)[None, :] <= (L - R + i)


@pytest.mark.parametrize("page_size", [1, 4, 16, 32, 64])
def test_paged_attention_equals_dense_numpy_on_gathered_tokens(oracle, page_size):
    wl = _wl(6, 2, 16)
    lens, ks = [37, 5, 64, 129, 16], [3, 4, 0, 2, 1]
    batch = synth.make_batch(wl, device="cpu", kv_lens=lens, k_per_seq=ks, seed=1, with_logits=False)
    pk = synth.paginate(batch.k_cache, batch.v_cache, lens, page_size, seed=page_size, extra_pages_per_seq=1)
    scale = 1.0 / math.sqrt(wl.D)
    out, lse = oracle.verify_attention_paged(
        batch.q.numpy(), pk.k_pages.numpy(), pk.v_pages.numpy(), batch.q_indptr.numpy(), pk.page_indptr.numpy(),
        pk.page_table.numpy(), pk.kv_len.numpy(), wl.Hq, wl.Hkv, wl.D, scale, oracle.F32, want_lse=True)
    assert np.isfinite(out).all()                     # the NaN in unused slots never enters
    qi = batch.q_indptr.numpy()
    for b, (L, k) in enumerate(zip(lens, ks)):
        kk, vv = _gathered(pk, b)
        ref = _dense(batch.q.numpy()[qi[b]:qi[b + 1]].astype(np.float64), kk, vv, 3, scale, _chain_visible(k + 1, L))
        np.testing.assert_allclose(out[qi[b]:qi[b + 1]], ref, rtol=0, atol=1e-12)
    # and the contiguous function on the original cache gives the same numbers
    flat = oracle.verify_attention(batch.q.numpy(), batch.k_cache.numpy(), batch.v_cache.numpy(), qi,
                                   batch.kv_indptr.numpy(), wl.Hq, wl.Hkv, wl.D, scale, oracle.F32)
    np.testing.assert_array_equal(out, flat)


def test_page_order_and_spare_pages_do_not_matter(oracle):
    wl = _wl(4, 4, 8, "bf16")
    lens, ks = [50, 33, 7], [2, 0, 4]
    batch = synth.make_batch(wl, device="cpu", kv_lens=lens, k_per_seq=ks, seed=2, with_logits=False)
    outs = []
    for seed, spare in ((0, 0), (1, 5), (2, 40)):
        pk = synth.paginate(batch.k_cache, batch.v_cache, lens, 16, seed=seed, spare_pages=spare)
        outs.append(oracle.verify_attention_paged(
            synth.to_host_array(batch.q), synth.to_host_array(pk.k_pages), synth.to_host_array(pk.v_pages),
            batch.q_indptr.numpy(), pk.page_indptr.numpy(), pk.page_table.numpy(), pk.kv_len.numpy(),
            wl.Hq, wl.Hkv, wl.D, 0.3, oracle.BF16))
    np.testing.assert_array_equal(outs[0], outs[1])
    np.testing.assert_array_equal(outs[0], outs[2])


def test_paged_tree_mask_equals_dense_numpy(oracle):
    wl = _wl(4, 2, 16)
    parents = [synth.caterpillar_parents(2, 2), [-1, 0, 0, 1, 1, 2], [-1]]
    tb = synth.make_tree_batch(wl, parents, device="cpu", kv_lens=[40, 6, 9], seed=3, with_logits=False)
    pk = synth.paginate(tb.k_cache, tb.v_cache, tb.kv_lens, 4, seed=5)
    mask = tb.tree_mask.numpy().view(np.uint64)
    out = oracle.verify_attention_paged(
        tb.q.numpy(), pk.k_pages.numpy(), pk.v_pages.numpy(), tb.q_indptr.numpy(), pk.page_indptr.numpy(),
        pk.page_table.numpy(), pk.kv_len.numpy(), wl.Hq, wl.Hkv, wl.D, 0.25, oracle.F32, tree_mask=mask)
    qi = tb.q_indptr.numpy()
    for b, par in enumerate(parents):
        R, L = len(par), tb.kv_lens[b]
        vis = np.ones((R, L), dtype=bool)
        for i in range(R):
            anc, j = {i}, i
            while par[j] >= 0:
                j = par[j]
                anc.add(j)
            for r in range(R):
                vis[i, L - R + r] = r in anc
        kk, vv = _gathered(pk, b)
        ref = _dense(tb.q.numpy()[qi[b]:qi[b + 1]].astype(np.float64), kk, vv, 2, 0.25, vis)
        np.testing.assert_allclose(out[qi[b]:qi[b + 1]], ref, rtol=0, atol=1e-12)


def test_bad_page_tables_are_data_errors(oracle):
    wl = _wl(2, 1, 8)
    batch = synth.make_batch(wl, device="cpu", kv_lens=[20], k_per_seq=[1], seed=4, with_logits=False)
    pk = synth.paginate(batch.k_cache, batch.v_cache, [20], 8, seed=0)
    args = lambda table, kv_len: (batch.q.numpy(), pk.k_pages.numpy(), pk.v_pages.numpy(), batch.q_indptr.numpy(),
                                  pk.page_indptr.numpy(), table, kv_len, wl.Hq, wl.Hkv, wl.D, 0.3, oracle.F32)
    bad = pk.page_table.numpy().copy()
    bad[1] = pk.num_pages
    with pytest.raises(RuntimeError):
        oracle.verify_attention_paged(*args(bad, pk.kv_len.numpy()))
    with pytest.raises(RuntimeError):          # more tokens than the sequence's pages hold
        oracle.verify_attention_paged(*args(pk.page_table.numpy(), np.array([25], dtype=np.int32)))


def _commit_case(wl, parents, lens, page_size, seed):
    tb = synth.make_tree_batch(wl, parents, device="cpu", kv_lens=lens, seed=seed, with_logits=False)
    pk = synth.paginate(tb.k_cache, tb.v_cache, tb.kv_lens, page_size, seed=seed, extra_pages_per_seq=1)
    return tb, pk


def test_chain_commit_only_cuts_the_length(oracle):
    wl = _wl(2, 2, 8)
    ks = [4, 3, 0, 2]
    tb, pk = _commit_case(wl, [list(range(-1, k)) for k in ks], [30, 9, 5, 17], 4, 6)
    k0, v0 = pk.k_pages.numpy().copy(), pk.v_pages.numpy().copy()
    kp, vp, kv_len = k0.copy(), v0.copy(), pk.kv_len.numpy().copy()
    n = np.array([2, 3, 0, 0], dtype=np.int32)
    oracle.commit_accepted_paged(kp, vp, tb.q_indptr.numpy(), pk.page_indptr.numpy(), pk.page_table.numpy(),
                                 kv_len, n, oracle.F32)
    np.testing.assert_array_equal(kp.view(np.uint32), k0.view(np.uint32))     # nothing moves in a chain
    np.testing.assert_array_equal(vp.view(np.uint32), v0.view(np.uint32))
    assert kv_len.tolist() == [30 - 4 + 2, 9 - 3 + 3, 5, 17 - 2]


def test_tree_commit_leaves_the_accepted_tokens_in_order(oracle):
    """After the commit the sequence reads: old tokens, last committed token, accepted nodes in
    path order; a new query over it attends exactly as over a cache built from those tokens."""
    wl = _wl(4, 2, 16)
    parents = [synth.caterpillar_parents(3, 3), [-1, 0, 0, 2, 2, 4], [-1, 0], synth.caterpillar_parents(2, 2),
               synth.caterpillar_parents(3, 3)]
    lens = [50, 8, 2, 21, 33]
    tb, pk = _commit_case(wl, parents, lens, 4, 7)
    path = np.array([[1, 4, 9], [2, 4, 5], [-1, -1, -1], [1, -1, -1], [3, -1, -1]], dtype=np.int32)
    n = np.array([3, 3, 0, 1, 1], dtype=np.int32)
    ki = tb.kv_indptr.numpy()
    expect = []
    for b, par in enumerate(parents):       # from the contiguous original, by plain indexing
        R, L = len(par), lens[b]
        keep = list(range(L - R + 1)) + [L - R + int(r) for r in path[b][:n[b]]]
        expect.append((tb.k_cache.numpy()[ki[b]:ki[b + 1]][keep], tb.v_cache.numpy()[ki[b]:ki[b + 1]][keep]))
    kp, vp, kv_len = pk.k_pages.numpy().copy(), pk.v_pages.numpy().copy(), pk.kv_len.numpy().copy()
    oracle.commit_accepted_paged(kp, vp, tb.q_indptr.numpy(), pk.page_indptr.numpy(), pk.page_table.numpy(),
                                 kv_len, n, oracle.F32, path=path)
    after = synth.PagedKV(torch.from_numpy(kp), torch.from_numpy(vp), pk.page_indptr, pk.page_table,
                          torch.from_numpy(kv_len), pk.page_size)
    for b in range(len(parents)):
        assert kv_len[b] == lens[b] - len(parents[b]) + 1 + n[b]
        kk, vv = _gathered(after, b)
        np.testing.assert_array_equal(kk, expect[b][0].astype(np.float64))
        np.testing.assert_array_equal(vv, expect[b][1].astype(np.float64))
    # one decode query per sequence over the committed cache == the contiguous function on `expect`
    gen = torch.Generator().manual_seed(0)
    q = torch.randn((len(parents), wl.Hq, wl.D), generator=gen).numpy()
    qi = np.arange(len(parents) + 1, dtype=np.int32)
    got = oracle.verify_attention_paged(q, kp, vp, qi, pk.page_indptr.numpy(), pk.page_table.numpy(), kv_len,
                                        wl.Hq, wl.Hkv, wl.D, 0.25, oracle.F32)
    flat_k = np.concatenate([e[0] for e in expect])
    flat_v = np.concatenate([e[1] for e in expect])
    kvi = np.concatenate([[0], np.cumsum([e[0].shape[0] for e in expect])]).astype(np.int64)
    ref = oracle.verify_attention(q, flat_k, flat_v, qi, kvi, wl.Hq, wl.Hkv, wl.D, 0.25, oracle.F32)
    np.testing.assert_array_equal(got, ref)


def test_commit_rejects_paths_that_are_not_increasing_rows(oracle):
    wl = _wl(2, 2, 8)
    tb, pk = _commit_case(wl, [[-1, 0, 0, 1]], [12], 4, 8)
    for bad_path, n in (([[2, 1, -1]], 2), ([[4, -1, -1]], 1), ([[0, -1, -1]], 1)):
        with pytest.raises(RuntimeError):
            oracle.commit_accepted_paged(pk.k_pages.numpy().copy(), pk.v_pages.numpy().copy(), tb.q_indptr.numpy(),
                                         pk.page_indptr.numpy(), pk.page_table.numpy(), pk.kv_len.numpy().copy(),
                                         np.array([n], dtype=np.int32), oracle.F32,
                                         path=np.array(bad_path, dtype=np.int32))
