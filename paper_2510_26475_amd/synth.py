"""Seeded synthetic inputs for the speculative-decoding verify step.

This module only draws random inputs of the right shapes; it holds none of the
method's arithmetic (no softmax, no acceptance test, no attention) and is the one
module the HIP path's tests/bench and the CPU oracle's tests both use.

The inputs stand in for the paper's RL rollouts (math datasets, 8K maximum response,
skewed lengths: Section 4.1 and the evaluation set-up): only shapes, length mixes and
logit statistics are imitated.

Recipe
------
* lengths ``L_b`` (cached tokens, the k_b+1 new ones included): uniform integers or a
  clipped log-normal, per workload;
* Q, K, V ~ N(0,1), rounded to the storage dtype;
* target logits ~ N(0, 3^2); drafter logits = target + N(0, sigma^2), both formed in
  fp32 and then rounded to the storage dtype;
* drafted tokens are exact samples from softmax(stored drafter logits / T), drawn with
  the Gumbel-max trick (argmax of logits/T + Gumbel noise), so the generator needs no
  softmax of its own;
* uniforms ~ U[0,1) in fp32, supplied to the sampler.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional, Sequence

import torch


@dataclass
class Workload:
    """One named verify-step workload."""
    name: str
    B: int
    k: int                      # drafted tokens per sequence (max when ragged_k)
    Hq: int
    Hkv: int
    D: int
    V: int
    dtype: str                  # "f32" or "bf16"
    len_dist: str               # "uniform" or "lognormal"
    len_lo: int
    len_hi: int
    len_median: float = 0.0     # lognormal only
    len_sigma: float = 0.0      # lognormal only
    sigma: float = 1.0          # drafter noise
    ragged_k: bool = False      # k_b ~ U{0..k}
    sigma_range: Optional[tuple] = None   # per-sequence sigma ~ U[a,b]
    seed: int = 0
    temperature: float = 1.0


# The five workloads named by the baseline description (index = config number - 1).
WORKLOADS = {
    "tiny_f32": Workload("tiny_f32", B=4, k=4, Hq=4, Hkv=1, D=64, V=1024, dtype="f32",
                         len_dist="uniform", len_lo=64, len_hi=256, seed=0),
    "qwen3b_b64_k4": Workload("qwen3b_b64_k4", B=64, k=4, Hq=16, Hkv=2, D=128, V=151936,
                              dtype="bf16", len_dist="uniform", len_lo=512, len_hi=4096, seed=1),
    "qwen7b_b256_k3": Workload("qwen7b_b256_k3", B=256, k=3, Hq=28, Hkv=4, D=128, V=151936,
                               dtype="bf16", len_dist="lognormal", len_lo=256, len_hi=8192,
                               len_median=2048.0, len_sigma=0.75, seed=2),
    "qwen14b_sweep": Workload("qwen14b_sweep", B=256, k=4, Hq=40, Hkv=8, D=128, V=151936,
                              dtype="bf16", len_dist="uniform", len_lo=1024, len_hi=8192, seed=3),
    "qwen14b_ragged": Workload("qwen14b_ragged", B=1024, k=8, Hq=40, Hkv=8, D=128, V=151936,
                               dtype="bf16", len_dist="lognormal", len_lo=256, len_hi=8192,
                               len_median=3072.0, len_sigma=0.8, ragged_k=True,
                               sigma_range=(0.5, 2.0), seed=4),
}


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


@dataclass
class VerifyBatch:
    """Device-resident inputs of one verify step (layouts as the C boundary takes them)."""
    wl: Workload
    q: torch.Tensor               # [total_q, Hq, D]
    k_cache: torch.Tensor         # [total_kv, Hkv, D]
    v_cache: torch.Tensor         # [total_kv, Hkv, D]
    q_indptr: torch.Tensor        # [B+1] int32
    kv_indptr: torch.Tensor       # [B+1] int64
    target_logits: torch.Tensor   # [total_q, V]
    draft_logits: torch.Tensor    # [total_q - B, V]
    draft_tokens: torch.Tensor    # [total_q - B] int32
    u_accept: torch.Tensor        # [total_q - B] f32
    u_final: torch.Tensor         # [B] f32
    k_per_seq: list = field(default_factory=list)
    kv_lens: list = field(default_factory=list)

    @property
    def total_q(self) -> int:
        return int(self.q.shape[0])

    @property
    def total_kv(self) -> int:
        return int(self.k_cache.shape[0])

    @property
    def max_k(self) -> int:
        return max(self.k_per_seq) if self.k_per_seq else 0

    @property
    def max_kv_len(self) -> int:
        return max(self.kv_lens)


def draw_lengths(wl: Workload, gen: torch.Generator) -> list:
    """Per-sequence cached lengths L_b (CPU generator, so the lengths are device independent)."""
    if wl.len_dist == "uniform":
        L = torch.randint(wl.len_lo, wl.len_hi + 1, (wl.B,), generator=gen)
    elif wl.len_dist == "lognormal":
        z = torch.randn(wl.B, generator=gen, dtype=torch.float64)
        L = torch.exp(math.log(wl.len_median) + wl.len_sigma * z).round().to(torch.int64)
        L = L.clamp(wl.len_lo, wl.len_hi)
    else:
        raise ValueError(wl.len_dist)
    return [int(x) for x in L.tolist()]


def draw_k(wl: Workload, gen: torch.Generator) -> list:
    if wl.ragged_k:
        return [int(x) for x in torch.randint(0, wl.k + 1, (wl.B,), generator=gen).tolist()]
    return [wl.k] * wl.B


def _randn(shape, gen, device, dtype=torch.float32, chunk_rows: int = 1 << 16):
    """Standard normal tensor, drawn in row chunks to bound the fp32 scratch."""
    out = torch.empty(shape, device=device, dtype=dtype)
    rows = shape[0]
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        out[r0:r1] = torch.randn((r1 - r0,) + tuple(shape[1:]), generator=gen, device=device,
                                 dtype=torch.float32).to(dtype)
    return out


def make_logits(n_target_rows: int, draft_row_sigma: torch.Tensor, draft_src_rows: torch.Tensor,
                V: int, dtype: torch.dtype, gen: torch.Generator, device,
                chunk_rows: int = 512):
    """target ~ N(0,9); draft[r] = target[draft_src_rows[r]] + sigma[r] * N(0,1); fp32 then rounded."""
    n_draft = int(draft_src_rows.numel())
    target = torch.empty((n_target_rows, V), device=device, dtype=dtype)
    draft = torch.empty((n_draft, V), device=device, dtype=dtype)
    src_pos = {int(s): i for i, s in enumerate(draft_src_rows.tolist())}
    for r0 in range(0, n_target_rows, chunk_rows):
        r1 = min(n_target_rows, r0 + chunk_rows)
        t32 = 3.0 * torch.randn((r1 - r0, V), generator=gen, device=device, dtype=torch.float32)
        target[r0:r1] = t32.to(dtype)
        rows = [r for r in range(r0, r1) if r in src_pos]
        if rows:
            local = torch.tensor([r - r0 for r in rows], device=device)
            dpos = torch.tensor([src_pos[r] for r in rows], device=device)
            noise = torch.randn((len(rows), V), generator=gen, device=device, dtype=torch.float32)
            sig = draft_row_sigma.to(device)[dpos].unsqueeze(1)
            draft[dpos] = (t32[local] + sig * noise).to(dtype)
    return target, draft


def sample_draft_tokens(draft_logits: torch.Tensor, temperature: float, gen: torch.Generator,
                        chunk_rows: int = 512) -> torch.Tensor:
    """x ~ softmax(draft_logits / T) through Gumbel-max (no softmax evaluated)."""
    n, V = draft_logits.shape
    out = torch.empty((n,), device=draft_logits.device, dtype=torch.int32)
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        u = torch.rand((r1 - r0, V), generator=gen, device=draft_logits.device, dtype=torch.float64)
        u = u.clamp_min(1e-300)
        gumbel = -torch.log(-torch.log(u))
        score = draft_logits[r0:r1].to(torch.float64) / float(temperature) + gumbel
        out[r0:r1] = score.argmax(dim=1).to(torch.int32)
    return out


def make_batch(wl: Workload, device="cpu", kv_lens: Optional[Sequence[int]] = None,
               k_per_seq: Optional[Sequence[int]] = None, seed: Optional[int] = None,
               with_attention: bool = True, with_logits: bool = True) -> VerifyBatch:
    """Draw every input of one verify step for workload ``wl`` on ``device``.

    The lengths and draft counts come from a CPU generator (same on every device); tensor
    values come from a generator on ``device`` (the oracle is always handed the same bytes
    the HIP path got, copied to the host).
    """
    seed = wl.seed if seed is None else seed
    cgen = torch.Generator(device="cpu").manual_seed(seed)
    kv_lens = list(kv_lens) if kv_lens is not None else draw_lengths(wl, cgen)
    k_per_seq = list(k_per_seq) if k_per_seq is not None else draw_k(wl, cgen)
    B = len(kv_lens)
    assert len(k_per_seq) == B
    for L, k in zip(kv_lens, k_per_seq):
        assert L >= k + 1, "a sequence's cache must hold its k+1 new tokens"
    if wl.sigma_range is not None:
        a, b = wl.sigma_range
        sig_seq = a + (b - a) * torch.rand(B, generator=cgen, dtype=torch.float32)
    else:
        sig_seq = torch.full((B,), float(wl.sigma), dtype=torch.float32)

    dgen = torch.Generator(device=device).manual_seed(seed + 1000003)
    dt = torch_dtype(wl.dtype)
    q_indptr = [0]
    kv_indptr = [0]
    for L, k in zip(kv_lens, k_per_seq):
        q_indptr.append(q_indptr[-1] + k + 1)
        kv_indptr.append(kv_indptr[-1] + L)
    total_q, total_kv = q_indptr[-1], kv_indptr[-1]

    if with_attention:
        q = _randn((total_q, wl.Hq, wl.D), dgen, device, dt)
        k_cache = _randn((total_kv, wl.Hkv, wl.D), dgen, device, dt)
        v_cache = _randn((total_kv, wl.Hkv, wl.D), dgen, device, dt)
    else:
        q = torch.empty((total_q, wl.Hq, wl.D), device=device, dtype=dt)
        k_cache = torch.empty((0, wl.Hkv, wl.D), device=device, dtype=dt)
        v_cache = torch.empty((0, wl.Hkv, wl.D), device=device, dtype=dt)

    n_draft = total_q - B
    if with_logits:
        src_rows, row_sigma = [], []
        for b, k in enumerate(k_per_seq):
            for i in range(k):
                src_rows.append(q_indptr[b] + i)
                row_sigma.append(float(sig_seq[b]))
        src_rows_t = torch.tensor(src_rows, dtype=torch.int64)
        row_sigma_t = torch.tensor(row_sigma, dtype=torch.float32)
        target, draft = make_logits(total_q, row_sigma_t, src_rows_t, wl.V, dt, dgen, device)
        draft_tokens = sample_draft_tokens(draft, wl.temperature, dgen)
    else:
        target = torch.empty((total_q, 0), device=device, dtype=dt)
        draft = torch.empty((n_draft, 0), device=device, dtype=dt)
        draft_tokens = torch.zeros((n_draft,), device=device, dtype=torch.int32)
    u_accept = torch.rand((n_draft,), generator=dgen, device=device, dtype=torch.float32)
    u_final = torch.rand((B,), generator=dgen, device=device, dtype=torch.float32)

    return VerifyBatch(
        wl=wl, q=q, k_cache=k_cache, v_cache=v_cache,
        q_indptr=torch.tensor(q_indptr, dtype=torch.int32, device=device),
        kv_indptr=torch.tensor(kv_indptr, dtype=torch.int64, device=device),
        target_logits=target, draft_logits=draft, draft_tokens=draft_tokens,
        u_accept=u_accept, u_final=u_final, k_per_seq=k_per_seq, kv_lens=kv_lens)


@dataclass
class TreeBatch:
    """One verify step over trees of drafts.  Row 0 of a sequence is the root (the last committed
    token), the other rows are draft nodes in an order in which parents come first."""
    wl: Workload
    q: torch.Tensor               # [total_q, Hq, D]
    k_cache: torch.Tensor         # [total_kv, Hkv, D]
    v_cache: torch.Tensor         # [total_kv, Hkv, D]
    q_indptr: torch.Tensor        # [B+1] int32
    kv_indptr: torch.Tensor       # [B+1] int64
    parent: torch.Tensor          # [total_q] int32, local row of the parent (-1 for the root)
    tree_mask: torch.Tensor       # [total_q] int64 holding 64 mask bits: bit j = new token j visible
    target_logits: torch.Tensor   # [total_q, V]
    draft_logits: torch.Tensor    # [total_q, V]  row i: what row i's children were drawn from
    node_tokens: torch.Tensor     # [total_q] int32 (-1 for the root)
    u_accept: torch.Tensor        # [total_q] f32 (the root's entry is unused)
    u_final: torch.Tensor         # [B] f32
    parents_per_seq: list = field(default_factory=list)
    kv_lens: list = field(default_factory=list)

    @property
    def total_q(self) -> int:
        return int(self.q.shape[0])

    @property
    def total_kv(self) -> int:
        return int(self.k_cache.shape[0])

    @property
    def max_rows(self) -> int:
        return max(len(p) for p in self.parents_per_seq)

    @property
    def max_kv_len(self) -> int:
        return max(self.kv_lens)

    @property
    def max_depth(self) -> int:
        best = 0
        for par in self.parents_per_seq:
            depth = [0] * len(par)
            for i in range(1, len(par)):
                depth[i] = depth[par[i]] + 1
            best = max(best, max(depth))
        return best


def caterpillar_parents(depth: int, branch: int) -> list:
    """A main chain of `depth` draft nodes in which every node of the chain (and the root) has
    `branch` children: the first continues the chain, the others are leaves.  1 + depth*branch rows."""
    par = [-1]
    spine = 0
    for _ in range(depth):
        first = len(par)
        for _ in range(branch):
            par.append(spine)
        spine = first
    return par


def random_parents(n_nodes: int, gen: torch.Generator, max_children: int = 3) -> list:
    """A random tree: every node picks a parent among the earlier rows that still has room."""
    par = [-1]
    kids = [0]
    for i in range(1, n_nodes + 1):
        room = [j for j in range(i) if kids[j] < max_children]
        j = room[int(torch.randint(0, len(room), (1,), generator=gen))]
        par.append(j)
        kids[j] += 1
        kids.append(0)
    return par


def make_tree_batch(wl: Workload, parents_per_seq: Sequence[Sequence[int]], device="cpu",
                    kv_lens: Optional[Sequence[int]] = None, seed: Optional[int] = None,
                    with_attention: bool = True, with_logits: bool = True) -> TreeBatch:
    """Inputs of one tree verify step.  The children of a row are drawn independently from the
    softmax of that row's drafter logits (Gumbel-max, no softmax evaluated)."""
    seed = wl.seed if seed is None else seed
    cgen = torch.Generator(device="cpu").manual_seed(seed)
    B = len(parents_per_seq)
    if kv_lens is None:
        wl_b = Workload(**{**wl.__dict__, "B": B})
        kv_lens = draw_lengths(wl_b, cgen)
    kv_lens = [max(int(L), len(par)) for L, par in zip(kv_lens, parents_per_seq)]
    dgen = torch.Generator(device=device).manual_seed(seed + 1000003)
    dt = torch_dtype(wl.dtype)
    q_indptr, kv_indptr, parent, mask = [0], [0], [], []
    for L, par in zip(kv_lens, parents_per_seq):
        assert par[0] == -1 and len(par) <= 64
        q_indptr.append(q_indptr[-1] + len(par))
        kv_indptr.append(kv_indptr[-1] + L)
        bits = []
        for i, pi in enumerate(par):
            assert i == 0 or 0 <= pi < i
            bits.append((1 << i) | (bits[pi] if pi >= 0 else 0))
        parent.extend(par)
        mask.extend(b - (1 << 64) if b >= (1 << 63) else b for b in bits)
    total_q, total_kv = q_indptr[-1], kv_indptr[-1]
    if with_attention:
        q = _randn((total_q, wl.Hq, wl.D), dgen, device, dt)
        k_cache = _randn((total_kv, wl.Hkv, wl.D), dgen, device, dt)
        v_cache = _randn((total_kv, wl.Hkv, wl.D), dgen, device, dt)
    else:
        q = torch.empty((total_q, wl.Hq, wl.D), device=device, dtype=dt)
        k_cache = torch.empty((0, wl.Hkv, wl.D), device=device, dtype=dt)
        v_cache = torch.empty((0, wl.Hkv, wl.D), device=device, dtype=dt)
    parent_t = torch.tensor(parent, dtype=torch.int32, device=device)
    if with_logits:
        rows = torch.arange(total_q, dtype=torch.int64)
        sig = torch.full((total_q,), float(wl.sigma), dtype=torch.float32)
        target, draft = make_logits(total_q, sig, rows, wl.V, dt, dgen, device)
        # the token of row i comes from the drafter row of its parent
        base = torch.repeat_interleave(torch.tensor(q_indptr[:-1], dtype=torch.int64),
                                       torch.tensor([len(p) for p in parents_per_seq]))
        src = (base + torch.tensor(parent, dtype=torch.int64).clamp_min(0)).to(device)
        node_tokens = sample_draft_tokens(draft[src], wl.temperature, dgen)
        node_tokens[parent_t < 0] = -1
    else:
        target = torch.empty((total_q, 0), device=device, dtype=dt)
        draft = torch.empty((total_q, 0), device=device, dtype=dt)
        node_tokens = torch.zeros((total_q,), device=device, dtype=torch.int32)
    u_accept = torch.rand((total_q,), generator=dgen, device=device, dtype=torch.float32)
    u_final = torch.rand((B,), generator=dgen, device=device, dtype=torch.float32)
    return TreeBatch(
        wl=wl, q=q, k_cache=k_cache, v_cache=v_cache,
        q_indptr=torch.tensor(q_indptr, dtype=torch.int32, device=device),
        kv_indptr=torch.tensor(kv_indptr, dtype=torch.int64, device=device),
        parent=parent_t, tree_mask=torch.tensor(mask, dtype=torch.int64, device=device),
        target_logits=target, draft_logits=draft, node_tokens=node_tokens,
        u_accept=u_accept, u_final=u_final, parents_per_seq=[list(p) for p in parents_per_seq],
        kv_lens=list(kv_lens))


import numpy as _np  # noqa: E402  (index bookkeeping only)


def sub_batch(batch: VerifyBatch, seqs) -> VerifyBatch:
    """The sequences ``seqs`` of ``batch`` as a batch of their own (same bytes, same device)."""
    qi = batch.q_indptr.cpu().tolist()
    ki = batch.kv_indptr.cpu().tolist()
    q_rows, kv_rows, d_rows = [], [], []
    for b in seqs:
        q_rows += list(range(qi[b], qi[b + 1]))
        kv_rows += list(range(ki[b], ki[b + 1]))
        d_rows += list(range(qi[b] - b, qi[b + 1] - (b + 1)))
    dev = batch.q.device
    qr = torch.tensor(q_rows, device=dev, dtype=torch.long)
    kr = torch.tensor(kv_rows, device=dev, dtype=torch.long)
    dr = torch.tensor(d_rows, device=dev, dtype=torch.long)
    ks = [batch.k_per_seq[b] for b in seqs]
    ls = [batch.kv_lens[b] for b in seqs]
    has_kv = batch.k_cache.shape[0] > 0
    has_logits = batch.target_logits.shape[1] > 0
    return VerifyBatch(
        wl=batch.wl, q=batch.q[qr].contiguous(),
        k_cache=batch.k_cache[kr].contiguous() if has_kv else batch.k_cache,
        v_cache=batch.v_cache[kr].contiguous() if has_kv else batch.v_cache,
        q_indptr=torch.tensor(_np.concatenate([[0], _np.cumsum([k + 1 for k in ks])]),
                              dtype=torch.int32, device=dev),
        kv_indptr=torch.tensor(_np.concatenate([[0], _np.cumsum(ls)]), dtype=torch.int64, device=dev),
        target_logits=batch.target_logits[qr].contiguous() if has_logits else batch.target_logits[qr],
        draft_logits=batch.draft_logits[dr].contiguous() if has_logits else batch.draft_logits[dr],
        draft_tokens=batch.draft_tokens[dr].contiguous(), u_accept=batch.u_accept[dr].contiguous(),
        u_final=batch.u_final[torch.tensor(list(seqs), device=dev, dtype=torch.long)].contiguous(),
        k_per_seq=ks, kv_lens=ls)


def to_host_array(t: torch.Tensor):
    """numpy view of a tensor for the oracle: float32 as is, bf16 as uint16 bit patterns."""
    import numpy as np
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


@dataclass
class PagedKV:
    """A KV cache cut into pages of ``page_size`` tokens (layout only, no arithmetic)."""
    k_pages: torch.Tensor       # [num_pages, page_size, Hkv, D]
    v_pages: torch.Tensor
    page_indptr: torch.Tensor   # [B+1] int32: pages of sequence b in page_table
    page_table: torch.Tensor    # [sum pages] int32 physical page ids, token order within a sequence
    kv_len: torch.Tensor        # [B] int32 tokens held by sequence b
    page_size: int

    @property
    def num_pages(self) -> int:
        return int(self.k_pages.shape[0])


def paginate(k_cache: torch.Tensor, v_cache: torch.Tensor, kv_lens: Sequence[int], page_size: int,
             seed: int = 0, spare_pages: int = 3, extra_pages_per_seq: int = 0, poison: bool = True) -> PagedKV:
    """Scatters a contiguous cache [total_kv, Hkv, D] into pages handed out in a seeded random
    order (plus ``spare_pages`` owned by nobody and ``extra_pages_per_seq`` allocated but unused
    pages behind every sequence).  With ``poison`` every slot no token lives in holds NaN."""
    dev = k_cache.device
    gen = torch.Generator(device="cpu").manual_seed(seed + 77)
    pages_per_seq = [(int(L) + page_size - 1) // page_size + extra_pages_per_seq for L in kv_lens]
    total_pages = sum(pages_per_seq)
    num_pages = total_pages + spare_pages
    order = torch.randperm(num_pages, generator=gen)[:total_pages].to(torch.int32)
    page_indptr = torch.tensor(_np.concatenate([[0], _np.cumsum(pages_per_seq)]), dtype=torch.int32)
    shape = (num_pages, page_size) + tuple(k_cache.shape[1:])
    fill = float("nan") if poison else 0.0
    k_pages = torch.full(shape, fill, dtype=k_cache.dtype, device=dev)
    v_pages = torch.full(shape, fill, dtype=v_cache.dtype, device=dev)
    # destination slot (page * page_size + offset) of every cached token
    dst = []
    for b, L in enumerate(kv_lens):
        j = torch.arange(int(L), dtype=torch.int64)
        pg = order[int(page_indptr[b]) + j // page_size].to(torch.int64)
        dst.append(pg * page_size + j % page_size)
    dst = torch.cat(dst).to(dev)
    k_pages.view((num_pages * page_size,) + tuple(k_cache.shape[1:]))[dst] = k_cache
    v_pages.view((num_pages * page_size,) + tuple(v_cache.shape[1:]))[dst] = v_cache
    return PagedKV(k_pages=k_pages, v_pages=v_pages, page_indptr=page_indptr.to(dev), page_table=order.to(dev),
                   kv_len=torch.tensor([int(L) for L in kv_lens], dtype=torch.int32, device=dev), page_size=page_size)
