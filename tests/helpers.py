"""Test-side glue: run one verify batch through the HIP library and through the oracle."""
from __future__ import annotations

import math
import os
from contextlib import contextmanager

import numpy as np
import torch

from paper_2510_26475_amd import binding, synth


@contextmanager
def env_setting(name, value):
    """Set (or, with None, unset) one environment knob of the library for the duration."""
    old = os.environ.get(name)
    if value is None:
        os.environ.pop(name, None)
    else:
        os.environ[name] = str(value)
    binding.respec_reload_knobs()   # the library reads its environment once; tell it to look again
    try:
        yield
    finally:
        if old is None:
            os.environ.pop(name, None)
        else:
            os.environ[name] = old
        binding.respec_reload_knobs()


def attn_wgs(wgs):
    """Force the number of ranges the key tiles are split over (None = the default, four per
    compute unit).  Small counts put many sequences in one range, large counts cut every
    sequence into many partials."""
    return env_setting("RESPEC_ATTN_WGS", wgs)


def gpu_attention(batch: synth.VerifyBatch, sm_scale=None, want_lse=True, stream=None):
    wl = batch.wl
    sm_scale = 1.0 / math.sqrt(wl.D) if sm_scale is None else sm_scale
    B = len(batch.kv_lens)
    max_q = max(batch.k_per_seq) + 1
    dt = binding.RESPEC_F32 if wl.dtype == "f32" else binding.RESPEC_BF16
    ws_bytes = binding.respec_verify_attention_workspace_bytes(
        B, batch.total_q, batch.total_kv, max_q, batch.max_kv_len, wl.Hq, wl.Hkv, wl.D, dt)
    assert ws_bytes > 0
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=batch.q.device)
    out = torch.full_like(batch.q, float("nan"))
    lse = torch.full((batch.total_q, wl.Hq), float("nan"), dtype=torch.float32,
                     device=batch.q.device) if want_lse else None
    binding.respec_verify_attention(batch.q, batch.k_cache, batch.v_cache, batch.q_indptr,
                                    batch.kv_indptr, out, lse, max_q, batch.max_kv_len, sm_scale,
                                    ws, stream=stream)
    torch.cuda.synchronize()
    return out, lse


def oracle_attention(oracle, batch: synth.VerifyBatch, sm_scale=None, n_threads=0):
    wl = batch.wl
    sm_scale = 1.0 / math.sqrt(wl.D) if sm_scale is None else sm_scale
    dt = oracle.F32 if wl.dtype == "f32" else oracle.BF16
    return oracle.verify_attention(
        synth.to_host_array(batch.q), synth.to_host_array(batch.k_cache),
        synth.to_host_array(batch.v_cache), batch.q_indptr.cpu().numpy(),
        batch.kv_indptr.cpu().numpy(), wl.Hq, wl.Hkv, wl.D, float(np.float32(sm_scale)), dt,
        want_lse=True, n_threads=n_threads)


sub_batch = synth.sub_batch


_SAMPLER_WORKSPACES = {}


def sampler_workspace(B, V, dtype_code, device):
    """The sampler's mailbox workspace: zero once, then reused by every later call (the
    library keeps it consistent from call to call)."""
    need = binding.respec_rejection_sample_workspace_bytes(B, B, V, dtype_code)
    key = (str(device), B)
    ws = _SAMPLER_WORKSPACES.get(key)
    if ws is None or ws.numel() < need:
        ws = torch.zeros(need, dtype=torch.uint8, device=device)
        _SAMPLER_WORKSPACES[key] = ws
    return ws


def sampler_split(split):
    """Force the number of work-groups that share a sequence (None: the library's choice)."""
    return env_setting("RESPEC_SAMPLER_SPLIT", split)


def gpu_sample(batch: synth.VerifyBatch, temperature=None, max_k=None, stream=None, workspace="shared"):
    wl = batch.wl
    T = wl.temperature if temperature is None else temperature
    B = len(batch.k_per_seq)
    max_k = batch.max_k if max_k is None else max_k
    dev = batch.target_logits.device
    toks = torch.full((B, max_k + 1), -7, dtype=torch.int32, device=dev)
    n = torch.full((B,), -7, dtype=torch.int32, device=dev)
    flags = torch.full((B,), -7, dtype=torch.int32, device=dev)
    if isinstance(workspace, str):
        dt = binding.RESPEC_F32 if batch.target_logits.dtype == torch.float32 else binding.RESPEC_BF16
        workspace = sampler_workspace(B, batch.target_logits.shape[1], dt, dev)
    binding.respec_rejection_sample(batch.target_logits, batch.draft_logits, batch.draft_tokens,
                                    batch.q_indptr, batch.u_accept, batch.u_final, toks, n, flags,
                                    max_k, T, workspace=workspace, stream=stream)
    torch.cuda.synchronize()
    return toks.cpu().numpy(), n.cpu().numpy(), flags.cpu().numpy()


def oracle_sample(oracle, batch: synth.VerifyBatch, temperature=None, max_k=None, n_threads=0):
    wl = batch.wl
    T = wl.temperature if temperature is None else temperature
    max_k = batch.max_k if max_k is None else max_k
    dt = oracle.F32 if wl.dtype == "f32" else oracle.BF16
    n_draft = batch.total_q - len(batch.k_per_seq)
    return oracle.rejection_sample(
        synth.to_host_array(batch.target_logits),
        synth.to_host_array(batch.draft_logits) if n_draft else None,
        batch.draft_tokens.cpu().numpy() if n_draft else None, batch.q_indptr.cpu().numpy(),
        batch.u_accept.cpu().numpy() if n_draft else None, batch.u_final.cpu().numpy(), max_k, T,
        dt, n_threads=n_threads)


def check_bf16_attention_rows(got: np.ndarray, ref: np.ndarray, rms_bound: float = 2.5e-3):
    """Element-wise bounds of a bf16 attention output [rows, heads, D] against the fp64 oracle.

    * absolute, the stated tolerance: 2e-2;
    * relative to the row: |err| <= 2^-7 * max|ref row| + 1e-3.  The output is rounded to bf16
      (half an ulp: at most 2^-8 of the element's magnitude) and so are the probabilities before
      the second product (2^-9 each, averaging over the keys); the largest absolute errors
      therefore sit in rows whose outputs are large, i.e. rows that see few keys or one dominant
      key (outputs of magnitude 2-4 round by up to 0.008-0.016), not in the long contexts;
    * rms over everything: 2.5e-3.
    """
    err = np.abs(got - ref)
    assert err.max() <= 2e-2, f"max abs err {err.max():.3e} > 2e-2"
    row_max = np.abs(ref).max(axis=-1, keepdims=True)
    excess = err - (2.0 ** -7 * row_max + 1e-3)
    assert excess.max() <= 0.0, (f"row-relative bound exceeded by {excess.max():.3e} at "
                                 f"{np.unravel_index(np.argmax(excess), excess.shape)}")
    rms = math.sqrt(float((err ** 2).mean()))
    assert rms <= rms_bound, f"rms err {rms:.3e}"
    return float(err.max())


def expected_flag_rate(V: int, logit_sigma: float = 3.0, eps: float = 1e-6) -> float:
    """Expected share of boundary draws for rows of V iid N(0, logit_sigma^2) logits.

    A draw is flagged when u*Z lies within eps*Z of an edge of the chosen token's CDF cell: for a
    token of mass w that happens with probability min(w, 2 eps), so the rate is
    sum_x min(w_x, 2 eps).  With w = e^z / (V e^{sigma^2/2}) the tokens above the threshold
    z* = ln(2 eps V) + sigma^2/2 contribute 2 eps each and the others their (lognormal) mass.
    (The accept tests add 2 eps per test, which is nothing.)  V = 151,936 and sigma = 3 give 0.07.
    """
    from scipy.stats import norm
    zs = math.log(2 * eps * V) + logit_sigma ** 2 / 2
    above = V * norm.sf(zs / logit_sigma)
    below_mass = norm.cdf((zs - logit_sigma ** 2) / logit_sigma)
    return min(1.0, 2 * eps * above + below_mass)


def flag_bound(B: int, V: int, logit_sigma: float = 3.0) -> float:
    """Mean plus four standard deviations (and one) of the number of boundary draws among B."""
    r = expected_flag_rate(V, logit_sigma)
    return B * r + 4.0 * math.sqrt(B * r * (1 - r)) + 1.0


def compare_sampler(gpu, ref):
    """Exact equality of tokens and counts on unflagged sequences; returns the boundary tally."""
    g_t, g_n, g_f = gpu
    r_t, r_n, r_f = ref
    flagged = r_f != 0
    same = (g_n == r_n) & (g_t == r_t).all(axis=1)
    bad = np.flatnonzero(~same & ~flagged)
    assert bad.size == 0, (
        f"{bad.size} unflagged sequences differ, first b={bad[0]}: gpu n={g_n[bad[0]]} "
        f"tokens={g_t[bad[0]].tolist()} vs oracle n={r_n[bad[0]]} tokens={r_t[bad[0]].tolist()}")
    return {"flagged": int(flagged.sum()), "flagged_mismatch": int((~same & flagged).sum()),
            "gpu_flagged": int((g_f != 0).sum()), "B": int(len(r_n))}


def gpu_tree_attention(tb: synth.TreeBatch, sm_scale=None, want_lse=True):
    wl = tb.wl
    sm_scale = 1.0 / math.sqrt(wl.D) if sm_scale is None else sm_scale
    B = len(tb.kv_lens)
    dt = binding.RESPEC_F32 if wl.dtype == "f32" else binding.RESPEC_BF16
    ws_bytes = binding.respec_verify_attention_workspace_bytes(
        B, tb.total_q, tb.total_kv, tb.max_rows, tb.max_kv_len, wl.Hq, wl.Hkv, wl.D, dt)
    assert ws_bytes > 0
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=tb.q.device)
    out = torch.full_like(tb.q, float("nan"))
    lse = torch.full((tb.total_q, wl.Hq), float("nan"), dtype=torch.float32,
                     device=tb.q.device) if want_lse else None
    binding.respec_verify_attention_tree(tb.q, tb.k_cache, tb.v_cache, tb.q_indptr, tb.kv_indptr,
                                         tb.tree_mask, out, lse, tb.max_rows, tb.max_kv_len, sm_scale, ws)
    torch.cuda.synchronize()
    return out, lse


def oracle_tree_attention(oracle, tb: synth.TreeBatch, sm_scale=None, n_threads=0):
    wl = tb.wl
    sm_scale = 1.0 / math.sqrt(wl.D) if sm_scale is None else sm_scale
    dt = oracle.F32 if wl.dtype == "f32" else oracle.BF16
    return oracle.verify_attention_tree(
        synth.to_host_array(tb.q), synth.to_host_array(tb.k_cache), synth.to_host_array(tb.v_cache),
        tb.q_indptr.cpu().numpy(), tb.kv_indptr.cpu().numpy(),
        tb.tree_mask.cpu().numpy().view(np.uint64), wl.Hq, wl.Hkv, wl.D, float(np.float32(sm_scale)), dt,
        want_lse=True, n_threads=n_threads)


def gpu_tree_sample(tb: synth.TreeBatch, temperature=None, max_depth=None):
    T = tb.wl.temperature if temperature is None else temperature
    B = len(tb.kv_lens)
    max_depth = tb.max_depth if max_depth is None else max_depth
    dev = tb.target_logits.device
    toks = torch.full((B, max_depth + 1), -7, dtype=torch.int32, device=dev)
    path = torch.full((B, max(max_depth, 1)), -7, dtype=torch.int32, device=dev)
    n = torch.full((B,), -7, dtype=torch.int32, device=dev)
    flags = torch.full((B,), -7, dtype=torch.int32, device=dev)
    binding.respec_tree_rejection_sample(tb.target_logits, tb.draft_logits, tb.node_tokens, tb.parent,
                                         tb.q_indptr, tb.u_accept, tb.u_final, toks, path, n, flags,
                                         tb.max_rows, max_depth, T)
    torch.cuda.synchronize()
    return toks.cpu().numpy(), path.cpu().numpy(), n.cpu().numpy(), flags.cpu().numpy()


def oracle_tree_sample(oracle, tb: synth.TreeBatch, temperature=None, max_depth=None, n_threads=0):
    T = tb.wl.temperature if temperature is None else temperature
    max_depth = tb.max_depth if max_depth is None else max_depth
    dt = oracle.F32 if tb.wl.dtype == "f32" else oracle.BF16
    return oracle.tree_rejection_sample(
        synth.to_host_array(tb.target_logits), synth.to_host_array(tb.draft_logits),
        tb.node_tokens.cpu().numpy(), tb.parent.cpu().numpy(), tb.q_indptr.cpu().numpy(),
        tb.u_accept.cpu().numpy(), tb.u_final.cpu().numpy(), max_depth, T, dt, n_threads=n_threads)


def compare_tree_sampler(gpu, ref):
    """Exact equality of tokens, path and counts on unflagged sequences; returns the boundary tally."""
    g_t, g_p, g_n, g_f = gpu
    r_t, r_p, r_n, r_f = ref
    flagged = r_f != 0
    same = (g_n == r_n) & (g_t == r_t).all(axis=1) & (g_p == r_p).all(axis=1)
    bad = np.flatnonzero(~same & ~flagged)
    assert bad.size == 0, (
        f"{bad.size} unflagged sequences differ, first b={bad[0]}: gpu n={g_n[bad[0]]} "
        f"tokens={g_t[bad[0]].tolist()} path={g_p[bad[0]].tolist()} vs oracle n={r_n[bad[0]]} "
        f"tokens={r_t[bad[0]].tolist()} path={r_p[bad[0]].tolist()}")
    return {"flagged": int(flagged.sum()), "flagged_mismatch": int((~same & flagged).sum()),
            "gpu_flagged": int((g_f != 0).sum()), "B": int(len(r_n))}


def sub_tree_batch(tb: synth.TreeBatch, seqs) -> synth.TreeBatch:
    """The sequences ``seqs`` of a tree batch as a batch of their own (attention inputs only)."""
    qi, ki = tb.q_indptr.cpu().tolist(), tb.kv_indptr.cpu().tolist()
    q_rows = [r for b in seqs for r in range(qi[b], qi[b + 1])]
    kv_rows = [r for b in seqs for r in range(ki[b], ki[b + 1])]
    dev = tb.q.device
    qr = torch.tensor(q_rows, device=dev, dtype=torch.long)
    kr = torch.tensor(kv_rows, device=dev, dtype=torch.long)
    pars = [tb.parents_per_seq[b] for b in seqs]
    lens = [tb.kv_lens[b] for b in seqs]
    return synth.TreeBatch(
        wl=tb.wl, q=tb.q[qr].contiguous(), k_cache=tb.k_cache[kr].contiguous(), v_cache=tb.v_cache[kr].contiguous(),
        q_indptr=torch.tensor(np.concatenate([[0], np.cumsum([len(p) for p in pars])]), dtype=torch.int32, device=dev),
        kv_indptr=torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int64, device=dev),
        parent=tb.parent[qr].contiguous(), tree_mask=tb.tree_mask[qr].contiguous(),
        target_logits=tb.target_logits[:0], draft_logits=tb.draft_logits[:0], node_tokens=tb.node_tokens[qr].contiguous(),
        u_accept=tb.u_accept[qr].contiguous(), u_final=tb.u_final[torch.tensor(list(seqs), device=dev)].contiguous(),
        parents_per_seq=pars, kv_lens=lens)


def gpu_paged_attention(batch, pk: synth.PagedKV, sm_scale=None, tree_mask=None, max_rows=None):
    """batch: a VerifyBatch or TreeBatch (q, q_indptr); the cache comes from ``pk``."""
    wl = batch.wl
    sm_scale = 1.0 / math.sqrt(wl.D) if sm_scale is None else sm_scale
    B = pk.kv_len.numel()
    max_rows = max_rows if max_rows is not None else int((batch.q_indptr[1:] - batch.q_indptr[:-1]).max())
    max_kv_len = int(pk.kv_len.max())
    dt = binding.RESPEC_F32 if wl.dtype == "f32" else binding.RESPEC_BF16
    ws_bytes = binding.respec_verify_attention_workspace_bytes(
        B, batch.total_q, pk.num_pages * pk.page_size, max_rows, max_kv_len, wl.Hq, wl.Hkv, wl.D, dt)
    assert ws_bytes > 0
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=batch.q.device)
    out = torch.full_like(batch.q, float("nan"))
    lse = torch.full((batch.total_q, wl.Hq), float("nan"), dtype=torch.float32, device=batch.q.device)
    binding.respec_verify_attention_paged(batch.q, pk.k_pages, pk.v_pages, batch.q_indptr, pk.page_indptr,
                                          pk.page_table, pk.kv_len, out, lse, max_rows, max_kv_len, sm_scale, ws,
                                          tree_mask=tree_mask)
    torch.cuda.synchronize()
    return out, lse


def oracle_paged_attention(oracle, batch, pk: synth.PagedKV, sm_scale=None, tree_mask=None, n_threads=0):
    wl = batch.wl
    sm_scale = 1.0 / math.sqrt(wl.D) if sm_scale is None else sm_scale
    dt = oracle.F32 if wl.dtype == "f32" else oracle.BF16
    return oracle.verify_attention_paged(
        synth.to_host_array(batch.q), synth.to_host_array(pk.k_pages), synth.to_host_array(pk.v_pages),
        batch.q_indptr.cpu().numpy(), pk.page_indptr.cpu().numpy(), pk.page_table.cpu().numpy(),
        pk.kv_len.cpu().numpy(), wl.Hq, wl.Hkv, wl.D, float(np.float32(sm_scale)), dt,
        tree_mask=None if tree_mask is None else tree_mask.cpu().numpy().view(np.uint64),
        want_lse=True, n_threads=n_threads)
