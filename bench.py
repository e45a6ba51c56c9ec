#!/usr/bin/env python3
"""Benchmark of the speculative-decoding verify step on one MI355X.

A "step" is one pass of the whole hot path over one synthetic batch: verify attention
(main kernel + split-KV combine, one layer) followed by rejection sampling.  All inputs
are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--sigma S]
                    [--tree DEPTHxBRANCH] [--page-size P] [--no-cpu-baseline] [--no-measure-depth]
    python bench.py --kd-rows N [--workload NAME] [--sigma S]
    python bench.py --sweep --workload qwen14b_sweep [--sweep-batches 64,256,...] [--sweep-ks 0,1,2,4,8]
    python bench.py --copy-probe 1024      # a copy of known size, to calibrate rocprofv3's byte counters

--tree times the tree-of-drafts variant of the step on the same workload (every sequence
drafts a main chain of DEPTH nodes with BRANCH candidates per position); the default is the
chain of k drafts the workload names.  --page-size scatters the KV cache over pages of P tokens
handed out in random order, runs attention through the page table and adds the commit of the
accepted tokens to the step.  --kd-rows times the drafter's reward-weighted distillation kernel
(not part of the verify step) on N row pairs of the workload's vocabulary and logits recipe.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2510_26475_amd import binding, synth  # noqa: E402

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth

# HBM bytes per launch of the attention main kernel from rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE runs, scaled by the same counters on a copy kernel of known size); the
# summaries are under profiles/.  None = not measured for that workload.
MEASURED_TRAFFIC_BYTES = {"qwen7b_b256_k3": 1.2285e9}
TRAFFIC_SOURCE = {"qwen7b_b256_k3": "profiles/verify_step_qwen7b_b256_k3.md (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE "
                                    "runs of this command, scaled by the same counters of `bench.py --copy-probe`; "
                                    "a constant copied from that summary, not a counter read in this run)"}


def attention_algorithmic_bytes(batch: synth.VerifyBatch) -> int:
    """K and V of every cached token once, Q in and O out once (split-KV partials excluded)."""
    wl = batch.wl
    esz = 4 if wl.dtype == "f32" else 2
    kv = batch.total_kv * wl.Hkv * wl.D * 2 * esz
    qo = 2 * batch.total_q * wl.Hq * wl.D * esz
    return kv + qo


def sampler_algorithmic_bytes(batch: synth.VerifyBatch, num_accepted) -> int:
    """Logit rows the method needs, once each: target rows 0..n_b, drafter rows 0..min(n_b,k_b-1)."""
    wl = batch.wl
    esz = 4 if wl.dtype == "f32" else 2
    rows = 0
    for n, k in zip(num_accepted, batch.k_per_seq):
        rows += (n + 1) + min(n + 1, k)
    return rows * wl.V * esz


def tree_sampler_algorithmic_bytes(tb: synth.TreeBatch, num_accepted, path) -> int:
    """Logit rows the method needs, once each: the target row of every node on the accepted path
    (root included) and the drafter row of those of them that have children."""
    esz = 4 if tb.wl.dtype == "f32" else 2
    rows = 0
    for b, par in enumerate(tb.parents_per_seq):
        has_child = set(par[1:])
        visited = [0] + [int(r) for r in path[b][:num_accepted[b]]]
        rows += len(visited) + sum(1 for r in visited if r in has_child)
    return rows * tb.wl.V * esz


def run_cpu_baseline_tree(tb: synth.TreeBatch, n_seqs: int):
    """The oracle's tree entry points timed on the host cores over the first n_seqs sequences."""
    import numpy as np

    import oracle  # test infrastructure: allowed here for the cpu_baseline leg only
    oracle.build()
    wl = tb.wl
    dt = oracle.F32 if wl.dtype == "f32" else oracle.BF16
    n_all = len(tb.parents_per_seq)
    threads = oracle.max_threads()

    def run(n, n_threads):
        n = max(1, min(n, n_all))
        rq, rk = int(tb.q_indptr[n]), int(tb.kv_indptr[n])
        h = dict(q=synth.to_host_array(tb.q[:rq]), k=synth.to_host_array(tb.k_cache[:rk]),
                 v=synth.to_host_array(tb.v_cache[:rk]), qi=tb.q_indptr[:n + 1].cpu().numpy(),
                 ki=tb.kv_indptr[:n + 1].cpu().numpy(), mask=tb.tree_mask[:rq].cpu().numpy().view(np.uint64),
                 t=synth.to_host_array(tb.target_logits[:rq]), d=synth.to_host_array(tb.draft_logits[:rq]),
                 tok=tb.node_tokens[:rq].cpu().numpy(), par=tb.parent[:rq].cpu().numpy(),
                 ua=tb.u_accept[:rq].cpu().numpy(), uf=tb.u_final[:n].cpu().numpy())
        t0 = time.perf_counter()
        oracle.verify_attention_tree(h["q"], h["k"], h["v"], h["qi"], h["ki"], h["mask"], wl.Hq, wl.Hkv, wl.D,
                                     float(np.float32(1.0 / math.sqrt(wl.D))), dt, n_threads=n_threads)
        t1 = time.perf_counter()
        _, _, n_acc, _ = oracle.tree_rejection_sample(h["t"], h["d"], h["tok"], h["par"], h["qi"], h["ua"], h["uf"],
                                                      tb.max_depth, wl.temperature, dt, n_threads=n_threads)
        t2 = time.perf_counter()
        return n, int((n_acc + 1).sum()), t1 - t0, t2 - t1

    n, emitted, ta, ts = run(n_seqs, 0)
    n1, emitted1, ta1, ts1 = run(n_seqs // max(1, threads), 1)
    return {
        "one_thread": {"value": emitted1 / (ta1 + ts1), "unit": "tokens/s", "sample": f"first {n1} sequences"},
        "value": emitted / (ta + ts), "unit": "tokens/s", "cores": threads, "kind": "oracle",
        "sample": f"first {n} of {n_all} sequences of the same workload, one attention layer + sampler, "
                  f"OpenMP over sequences",
        "attention_s": ta, "sampler_s": ts, "emitted_tokens": emitted,
    }


def run_cpu_baseline(batch: synth.VerifyBatch, n_seqs: int):
    """The oracle, as it stands, timed on the host cores over the first n_seqs sequences."""
    import numpy as np

    import oracle  # test infrastructure: allowed here for the cpu_baseline leg only
    oracle.build()
    n_seqs = min(n_seqs, len(batch.k_per_seq))
    sb = synth.sub_batch(batch, list(range(n_seqs)))
    wl = sb.wl
    dt = oracle.F32 if wl.dtype == "f32" else oracle.BF16
    host = dict(
        q=synth.to_host_array(sb.q), k=synth.to_host_array(sb.k_cache),
        v=synth.to_host_array(sb.v_cache), qi=sb.q_indptr.cpu().numpy(),
        ki=sb.kv_indptr.cpu().numpy(), t=synth.to_host_array(sb.target_logits),
        d=synth.to_host_array(sb.draft_logits), tok=sb.draft_tokens.cpu().numpy(),
        ua=sb.u_accept.cpu().numpy(), uf=sb.u_final.cpu().numpy())
    threads = oracle.max_threads()
    t0 = time.perf_counter()
    attn_out, attn_lse = oracle.verify_attention(host["q"], host["k"], host["v"], host["qi"], host["ki"], wl.Hq,
                                                 wl.Hkv, wl.D, float(np.float32(1.0 / math.sqrt(wl.D))), dt,
                                                 want_lse=True, n_threads=0)
    t1 = time.perf_counter()
    n_draft = sb.total_q - n_seqs
    toks, n, oflags = oracle.rejection_sample(
        host["t"], host["d"] if n_draft else None, host["tok"] if n_draft else None, host["qi"],
        host["ua"] if n_draft else None, host["uf"], sb.max_k, wl.temperature, dt, n_threads=0)
    t2 = time.perf_counter()
    emitted = int((n + 1).sum())
    # one thread, on the first sequences only (it is about `threads` times slower)
    n1 = max(1, min(n_seqs, n_seqs // max(1, threads)))
    s1 = synth.sub_batch(batch, list(range(n1)))
    h1 = dict(q=synth.to_host_array(s1.q), k=synth.to_host_array(s1.k_cache), v=synth.to_host_array(s1.v_cache),
              qi=s1.q_indptr.cpu().numpy(), ki=s1.kv_indptr.cpu().numpy(), t=synth.to_host_array(s1.target_logits),
              d=synth.to_host_array(s1.draft_logits), tok=s1.draft_tokens.cpu().numpy(),
              ua=s1.u_accept.cpu().numpy(), uf=s1.u_final.cpu().numpy())
    t3 = time.perf_counter()
    oracle.verify_attention(h1["q"], h1["k"], h1["v"], h1["qi"], h1["ki"], wl.Hq, wl.Hkv, wl.D,
                            float(np.float32(1.0 / math.sqrt(wl.D))), dt, n_threads=1)
    nd1 = s1.total_q - n1
    _, n_1, _ = oracle.rejection_sample(
        h1["t"], h1["d"] if nd1 else None, h1["tok"] if nd1 else None, h1["qi"],
        h1["ua"] if nd1 else None, h1["uf"], s1.max_k, wl.temperature, dt, n_threads=1)
    t4 = time.perf_counter()
    line = {
        "one_thread": {"value": int((n_1 + 1).sum()) / (t4 - t3), "unit": "tokens/s",
                       "sample": f"first {n1} sequences"},
        "value": emitted / (t2 - t0), "unit": "tokens/s", "cores": threads, "kind": "oracle",
        "sample": f"first {n_seqs} of {len(batch.k_per_seq)} sequences of the same workload, "
                  f"one attention layer + sampler, OpenMP over sequences",
        "attention_s": t1 - t0, "sampler_s": t2 - t1, "emitted_tokens": emitted,
    }
    return line, dict(n_seqs=n_seqs, rows=sb.total_q, out=attn_out, lse=attn_lse, tokens=toks, n=n, flags=oflags)


def parity_tally(ref, gpu_out, gpu_lse, gpu_toks, gpu_n, gpu_flags, bf16: bool):
    """The HIP path's results of the benchmarked launch against the oracle's, on the sequences the
    cpu_baseline leg walked (outside the timed region).  Tokens and counts must agree exactly on
    every sequence that neither side flags as a boundary draw; flagged ones are counted."""
    import numpy as np
    ns, rows = ref["n_seqs"], ref["rows"]
    gt, gn, gf = gpu_toks[:ns].cpu().numpy(), gpu_n[:ns].cpu().numpy(), gpu_flags[:ns].cpu().numpy()
    same = (gt == ref["tokens"]).all(axis=1) & (gn == ref["n"])
    flagged = (ref["flags"] != 0) | (gf != 0)
    err = np.abs(gpu_out[:rows].double().cpu().numpy() - ref["out"])
    row_ref = np.abs(ref["out"]).max(axis=-1, keepdims=True)
    lse_err = np.abs(gpu_lse[:rows].double().cpu().numpy() - ref["lse"])
    return {
        "sequences": int(ns), "oracle_flagged": int((ref["flags"] != 0).sum()), "gpu_flagged": int((gf != 0).sum()),
        "unflagged_mismatch": int((~same & ~flagged).sum()), "flagged_mismatch": int((~same & flagged).sum()),
        "attention_rows": int(rows), "attention_max_abs_err": float(err.max()),
        "attention_max_err_over_row_max": float((err / np.maximum(row_ref, 1e-30)).max()),
        "attention_tolerance": 2e-2 if bf16 else 1e-5, "lse_max_abs_err": float(lse_err.max()),
        "note": "oracle vs the HIP path on the same bytes; a boundary draw lies within 1e-6 of an accept "
                "threshold or of an edge of the chosen token's CDF cell",
    }


def run_kd(args, wl, dev):
    """respec_kd_rows on args.kd_rows row pairs: HIP-event time of the row kernel's call, oracle beside it."""
    rows, V = args.kd_rows, wl.V
    g = torch.Generator(device=dev).manual_seed(wl.seed)
    tdt = torch.float32 if wl.dtype == "f32" else torch.bfloat16
    t32 = 3.0 * torch.randn((rows, V), generator=g, device=dev)
    target = t32.to(tdt)
    t32 += wl.sigma * torch.randn((rows, V), generator=g, device=dev)
    draft = t32.to(tdt)
    del t32
    w = 0.1 + 1.9 * torch.rand((rows,), generator=g, device=dev)
    dt = binding.RESPEC_F32 if wl.dtype == "f32" else binding.RESPEC_BF16
    ws = torch.empty(binding.respec_kd_rows_workspace_bytes(rows, V, dt), dtype=torch.uint8, device=dev)
    grad = torch.empty_like(draft)
    loss = torch.empty((rows,), dtype=torch.float32, device=dev)
    total = torch.empty((1,), dtype=torch.float64, device=dev)
    for _ in range(args.warmup):
        binding.respec_kd_rows(target, draft, w, grad, loss, total, ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        binding.respec_kd_rows(target, draft, w, grad, loss, total, ws)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    esz = 4 if wl.dtype == "f32" else 2
    algo = 3 * rows * V * esz   # both rows read once, the gradient written once
    line = {
        "metric": "logit rows/s of the reward-weighted KD row kernel (loss and gradient of the drafter's logits)",
        "value": rows / (ms * 1e-3), "unit": "rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": f"kd_rows on {rows} row pairs of {wl.name}", "rows": rows, "V": V, "sigma": wl.sigma,
                   "seed": wl.seed},
        "total_loss": float(total.item()),
        "roofline": {"kernel": "kd_stream_kernel", "bound": "hbm", "achieved": algo / (ms * 1e-3) / 1e9,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": algo / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": 2.925e9 if (rows == 2048 and V == 151936 and wl.dtype == "bf16") else None,
                     "note": "time per call (row kernel + the one-work-group finish kernel) by HIP events"},
    }
    if not args.no_cpu_baseline:
        import oracle  # test infrastructure: allowed here for the cpu_baseline leg only
        oracle.build()
        n = min(rows, 64)
        th, dh, wh = synth.to_host_array(target[:n]), synth.to_host_array(draft[:n]), w[:n].cpu().numpy()
        odt = oracle.F32 if wl.dtype == "f32" else oracle.BF16
        t0 = time.perf_counter()
        oracle.kd_rows(th, dh, wh, odt, n_threads=0)
        t1 = time.perf_counter()
        line["cpu_baseline"] = {"value": n / (t1 - t0), "unit": "rows/s", "cores": oracle.max_threads(),
                                "kind": "oracle", "sample": f"first {n} of {rows} row pairs, OpenMP over rows"}
    print(json.dumps(line))


def bench_verify(args, wl, dev, changed: bool, cpu_baseline: bool):
    """Times the verify step on workload `wl`; returns the JSON line as a dict."""
    tree = None
    if args.tree:
        depth, branch = (int(x) for x in args.tree.lower().split("x"))
        tree = synth.caterpillar_parents(depth, branch)
        cgen = torch.Generator(device="cpu").manual_seed(wl.seed)
        batch = synth.make_tree_batch(wl, [tree] * wl.B, device=dev, kv_lens=synth.draw_lengths(wl, cgen))
        B, max_q, max_out = wl.B, batch.max_rows, batch.max_depth
    else:
        batch = synth.make_batch(wl, device=dev)
        B = len(batch.k_per_seq)
        max_q = batch.max_k + 1
        max_out = batch.max_k
    dt = binding.RESPEC_F32 if wl.dtype == "f32" else binding.RESPEC_BF16
    ws_bytes = binding.respec_verify_attention_workspace_bytes(
        B, batch.total_q, batch.total_kv, max_q, batch.max_kv_len, wl.Hq, wl.Hkv, wl.D, dt)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    out = torch.empty_like(batch.q)
    lse = torch.empty((batch.total_q, wl.Hq), dtype=torch.float32, device=dev)
    toks = torch.empty((B, max_out + 1), dtype=torch.int32, device=dev)
    path = torch.empty((B, max(max_out, 1)), dtype=torch.int32, device=dev)
    n_acc = torch.empty((B,), dtype=torch.int32, device=dev)
    flags = torch.empty((B,), dtype=torch.int32, device=dev)
    sm_scale = 1.0 / math.sqrt(wl.D)
    # the sampler's mailbox workspace: zero before its first use, then left to the library
    samp_ws = torch.zeros(binding.respec_rejection_sample_workspace_bytes(B, batch.total_q, wl.V, dt),
                          dtype=torch.uint8, device=dev)

    turn = {"i": 0}
    paged = None
    if args.page_size:
        paged = synth.paginate(batch.k_cache, batch.v_cache, batch.kv_lens, args.page_size, seed=wl.seed,
                               spare_pages=64, poison=False)
        kv_len0 = paged.kv_len.clone()
    mask = batch.tree_mask if tree is not None else None

    if paged is not None:
        def attention():
            binding.respec_verify_attention_paged(batch.q, paged.k_pages, paged.v_pages, batch.q_indptr,
                                                  paged.page_indptr, paged.page_table, kv_len0, out, lse, max_q,
                                                  batch.max_kv_len, sm_scale, ws, tree_mask=mask)

        def commit():
            # the lengths are restored first so that every step commits the same verify result
            paged.kv_len.copy_(kv_len0)
            binding.respec_commit_accepted_paged(paged.k_pages, paged.v_pages, batch.q_indptr, paged.page_indptr,
                                                 paged.page_table, paged.kv_len, n_acc, batch.total_q, max_q,
                                                 path=path if tree is not None else None)
    else:
        # --rotate N: N copies of the large inputs (KV cache, logits) used in turn, so that no step
        # finds its data in the last-level cache from the step before (chain drafts only)
        n_sets = max(1, args.rotate) if tree is None else 1
        sets = [(batch.k_cache, batch.v_cache, batch.target_logits, batch.draft_logits)]
        for _ in range(n_sets - 1):
            sets.append(tuple(t.clone() for t in sets[0]))

        def commit():
            turn["i"] += 1

        if tree is not None:
            def attention():
                binding.respec_verify_attention_tree(batch.q, batch.k_cache, batch.v_cache, batch.q_indptr,
                                                     batch.kv_indptr, batch.tree_mask, out, lse, max_q,
                                                     batch.max_kv_len, sm_scale, ws)
        else:
            def attention():
                kc, vc = sets[turn["i"] % n_sets][:2]
                binding.respec_verify_attention(batch.q, kc, vc, batch.q_indptr,
                                                batch.kv_indptr, out, lse, max_q, batch.max_kv_len,
                                                sm_scale, ws)

    if tree is not None:
        def sampler():
            binding.respec_tree_rejection_sample(batch.target_logits, batch.draft_logits, batch.node_tokens,
                                                 batch.parent, batch.q_indptr, batch.u_accept, batch.u_final,
                                                 toks, path, n_acc, flags, max_q, max_out, wl.temperature)
    else:
        def sampler():
            tl, dl = sets[turn["i"] % n_sets][2:] if paged is None else (batch.target_logits, batch.draft_logits)
            binding.respec_rejection_sample(tl, dl,
                                            batch.draft_tokens, batch.q_indptr, batch.u_accept,
                                            batch.u_final, toks, n_acc, flags, batch.max_k,
                                            wl.temperature, workspace=samp_ws)

    for _ in range(args.warmup):
        attention()
        sampler()
        commit()
    torch.cuda.synchronize()

    # Timed region: exactly --steps steps.  An event record costs a few microseconds of stream
    # time, so only the main attention kernel is bracketed (the library records the two events
    # right around its launch, on the launch stream), and only on every --probe-every-th step.
    probe = max(1, args.probe_every)
    probes = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range((args.steps + probe - 1) // probe)]
    for a, b in probes:
        a.record()      # create the handles the library will re-record
        b.record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        if i % probe == 0:
            a, b = probes[i // probe]
            binding.respec_profile_mark_main(a, b)
        attention()
        sampler()
        commit()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / args.steps
    ms_main = sum(a.elapsed_time(b) for a, b in probes) / len(probes)

    # The other kernels' times come from a separate, fully instrumented pass after the timed
    # region (five events per step; its steps are slower for it and are not part of `value`).
    n_pass = min(args.steps, 10)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(n_pass)]
    for e4 in ev:
        e4[1].record()
        e4[4].record()
    torch.cuda.synchronize()
    for e4 in ev:
        e4[0].record()
        binding.respec_profile_mark_main(e4[4], e4[1])
        attention()
        e4[2].record()
        sampler()
        e4[3].record()
        commit()
        e4[5].record()
    torch.cuda.synchronize()
    ms_main_pass = sum(e4[4].elapsed_time(e4[1]) for e4 in ev) / n_pass
    ms_prep = sum(e4[0].elapsed_time(e4[4]) for e4 in ev) / n_pass
    ms_comb = sum(e4[1].elapsed_time(e4[2]) for e4 in ev) / n_pass
    ms_samp = sum(e4[2].elapsed_time(e4[3]) for e4 in ev) / n_pass
    ms_commit = sum(e4[3].elapsed_time(e4[5]) for e4 in ev) / n_pass if paged is not None else 0.0

    # a device copy of 1 GiB, timed live: what this device's memory system gives a trivial kernel
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * src.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst
    main_sorted = sorted(a.elapsed_time(b) for a, b in probes)
    layers = args.layers or {"qwen3b": 36, "qwen7b": 28, "qwen14b": 48}.get(wl.name.split("_")[0], 1)

    # Optional: the full-depth step measured instead of modelled.  Every layer gets a KV cache of
    # its own (same lengths, fresh random values, so no layer finds its cache in a cache), one
    # attention call per layer, then the sampler.  GEMMs, norms and the LM head stay outside.
    measured_depth = None
    kv_bytes_all_layers = layers * 2 * batch.k_cache.numel() * batch.k_cache.element_size()
    want_depth = args.measure_depth if args.measure_depth is not None else (
        kv_bytes_all_layers < 64e9 and not args.sweep)
    if want_depth and tree is None and paged is None:
        g2 = torch.Generator(device=dev).manual_seed(wl.seed + 1000)
        caches = [(batch.k_cache, batch.v_cache)]
        for _ in range(layers - 1):
            kc = torch.empty_like(batch.k_cache).normal_(generator=g2)
            vc = torch.empty_like(batch.v_cache).normal_(generator=g2)
            caches.append((kc, vc))

        def deep_step():
            for i, (kc, vc) in enumerate(caches):  # layers after the first reuse the first one's set-up
                call = binding.respec_verify_attention if i == 0 else binding.respec_verify_attention_next_layer
                call(batch.q, kc, vc, batch.q_indptr, batch.kv_indptr, out, lse, max_q, batch.max_kv_len,
                     sm_scale, ws)
            sampler()

        for _ in range(2):
            deep_step()
        torch.cuda.synchronize()
        n_deep = max(3, min(args.steps, 10))
        d0 = time.perf_counter()
        for _ in range(n_deep):
            deep_step()
        torch.cuda.synchronize()
        us_deep = (time.perf_counter() - d0) * 1e6 / n_deep
        measured_depth = {"layers": layers, "steps": n_deep, "us_per_step": us_deep,
                          "note": "MEASURED: one attention call per layer on a KV cache of its own (the first call sets up, the "
                                  "others reuse it: respec_verify_attention_next_layer), then the sampler; "
                                  "the forward's GEMMs are outside this path"}
        del caches

    n_host = n_acc.cpu().tolist()
    accepted = int(sum(n_host))
    emitted = accepted + B
    attn_bytes = attention_algorithmic_bytes(batch)
    esz = 4 if wl.dtype == "f32" else 2
    if tree is not None:
        samp_bytes = tree_sampler_algorithmic_bytes(batch, n_host, path.cpu().tolist())
        samp_all_rows = 2 * batch.total_q * wl.V * esz
    else:
        samp_bytes = sampler_algorithmic_bytes(batch, n_host)
        samp_all_rows = (batch.total_q + batch.total_q - B) * wl.V * esz
    achieved = attn_bytes / (ms_main * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get(wl.name) if not changed and tree is None and paged is None else None

    line = {
        # the headline workload carries the baseline's own wording of the metric: `value` is its
        # tokens/s part, `verify_step_us` and `roofline.frac` / `step_hbm_frac` the other two
        "metric": ("accepted tokens/s + verify-step us at B=256,k=3 (7B shapes); % HBM roofline"
                   if wl.name == "qwen7b_b256_k3" and not changed and tree is None and paged is None else
                   "accepted tokens/s of the SD verify step"),
        "metric_note": "tokens emitted per step = accepted drafts + 1 per sequence; a step = one attention layer "
                       "(set-up, main, combine) + rejection sampling",
        "value": emitted / (ms_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {
            "workload": (wl.name if tree is None else f"{wl.name}+tree{args.tree}") +
                        (f"+pages{args.page_size}" if paged is not None else ""),
            "kv_cache": "contiguous per sequence" if paged is None else
                        f"paged, {args.page_size} tokens per page, pages handed out in random order",
            "drafts": f"chain of k={wl.k}" if tree is None else
                      f"tree: chain of {depth} nodes, {branch} candidates per position, {len(tree)} rows per sequence",
            "B": B, "k": wl.k, "ragged_k": wl.ragged_k, "Hq": wl.Hq,
            "Hkv": wl.Hkv, "D": wl.D, "V": wl.V, "sigma": wl.sigma, "temperature": wl.temperature,
            "kv_len": f"{wl.len_dist}[{wl.len_lo},{wl.len_hi}]", "total_kv": batch.total_kv,
            "seed": wl.seed, "rotating_input_sets": args.rotate if (tree is None and paged is None) else 1,
        },
        "verify_step_us": ms_step * 1e3,
        "kernel_us": {"attention_before_main": ms_prep * 1e3, "attention_main": ms_main * 1e3, "attention_combine": ms_comb * 1e3,
                      "rejection_sample": ms_samp * 1e3, "commit_accepted": ms_commit * 1e3},
        "kernel_us_note": "attention_before_main: from an event ahead of the call to the start of the main kernel "
                          "(a launch gap; plus the set-up kernel for batches of more than 2048 sequences, whose "
                          "split is not built in the main kernel's prologue); "
                          "attention_main: HIP events around the launch on every %d-th step of the timed region; "
                          "the others (launch gaps included) and attention_main_instrumented_pass: a separate pass "
                          "of %d fully instrumented steps after it" % (probe, n_pass),
        "attention_main_instrumented_pass_us": ms_main_pass * 1e3,
        "accepted_drafts": accepted, "emitted_tokens": emitted,
        "emitted_per_seq": emitted / B,
        "accepted_drafts_per_s": accepted / (ms_step * 1e-3),
        "boundary_flagged": int((flags != 0).sum().item()),
        "algorithmic_bytes": {"attention": attn_bytes, "sampler_needed_rows": samp_bytes,
                              "sampler_all_rows": samp_all_rows},
        "step_hbm_frac": (attn_bytes + samp_bytes) / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "sampler_gbs": samp_bytes / (ms_samp * 1e-3) / 1e9,
        "t_attn_us": (ms_prep + ms_main_pass + ms_comb) * 1e3, "t_samp_us": ms_samp * 1e3,
        "tokens_per_s_kernels": emitted / ((ms_prep + ms_main_pass + ms_comb + ms_samp) * 1e-3),
        "modelled_full_depth": {"layers": layers, "note": "MODELLED, not measured: emitted / (layers * t_attn + t_samp)",
                                "tokens_per_s": emitted / ((layers * (ms_prep + ms_main_pass + ms_comb) + ms_samp) * 1e-3)},
        "measured_full_depth": (dict(measured_depth, tokens_per_s=emitted / (measured_depth["us_per_step"] * 1e-6))
                                if measured_depth else None),
        "attention_main_us_median_min": [main_sorted[len(main_sorted) // 2] * 1e3, main_sorted[0] * 1e3],
        "measured_copy_gbs": copy_gbs,
        "attention_frac_of_measured_copy": achieved / copy_gbs,
        "roofline": {
            "kernel": "attn_bf16_kernel" if wl.dtype == "bf16" else "attn_f32_kernel",
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
            "traffic_source": TRAFFIC_SOURCE.get(wl.name) if traffic is not None else None,
        },
    }
    if cpu_baseline:
        if tree is not None:
            line["cpu_baseline"] = run_cpu_baseline_tree(batch, args.cpu_seqs)
        else:
            line["cpu_baseline"], ref = run_cpu_baseline(batch, args.cpu_seqs)
            # the benchmarked launch's own outputs against the oracle's (first input set)
            turn["i"] = 0
            attention()
            sampler()
            torch.cuda.synchronize()
            line["parity"] = parity_tally(ref, out, lse, toks, n_acc, flags, wl.dtype == "bf16")
        if paged is not None:
            line["cpu_baseline"]["note"] = ("timed on the oracle's contiguous-cache functions: its paged form "
                                            "gathers a sequence's pages and calls them")
    return line


def solver_table(rows, ratios=(0.02, 0.05, 0.1, 0.25)):
    """The Solver's table from a sweep: for every profiled batch size and every drafter cost
    (one drafter step = ratio x the plain decoding step at that batch), the draft length that
    respec_solver_pick chooses and the speedup it predicts.  Times are the MODELLED full-depth
    step, layers x attention + sampler (this path has no GEMMs)."""
    pts = [(r["B"], r["k"], r["layers"] * r["t_attn_us"] + r["t_samp_us"], r["emitted_per_seq"]) for r in rows]
    table = []
    for B in sorted({r["B"] for r in rows}):
        decode_us = next(t for (b, k, t, e) in pts if b == B and k == 0)
        for ratio in ratios:
            best, speedup, cost = binding.respec_solver_pick(pts, B, ratio * decode_us, 0.0)
            table.append({"B": B, "draft_cost_ratio": ratio, "best_k": best, "predicted_speedup": speedup,
                          "cost_us_per_token": cost})
    return table


def run_sweep(args, wl, dev):
    """The B x k sweep of the large-batch workload: one verify step timed per (B, k), k = 0 being
    plain decoding (one row per sequence, one token per step).  Prints one JSON line whose
    `sweep` list holds a compact record per point."""
    import dataclasses
    import gc
    Bs = [int(x) for x in args.sweep_batches.split(",")]
    ks = [int(x) for x in args.sweep_ks.split(",")]
    rows = []
    for B in Bs:
        for k in ks:
            w2 = dataclasses.replace(wl, B=B, k=k)
            line = bench_verify(args, w2, dev, True, False)
            rows.append({
                "B": B, "k": k, "verify_step_us": line["verify_step_us"], "t_attn_us": line["t_attn_us"],
                "t_samp_us": line["t_samp_us"], "attention_main_us": line["kernel_us"]["attention_main"],
                "emitted_per_seq": line["emitted_per_seq"], "tokens_per_s": line["value"],
                "accepted_drafts_per_s": line["accepted_drafts_per_s"],
                "attention_frac": line["roofline"]["frac"], "step_hbm_frac": line["step_hbm_frac"],
                "total_kv": line["config"]["total_kv"],
                "modelled_full_depth_tokens_per_s": line["modelled_full_depth"]["tokens_per_s"],
                "layers": line["modelled_full_depth"]["layers"],
            })
            print("sweep point", json.dumps(rows[-1]), file=sys.stderr, flush=True)
            del line
            gc.collect()
            torch.cuda.empty_cache()
    out = {"metric": "accepted tokens/s of the SD verify step over the B x k sweep", "unit": "tokens/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "dtype": wl.dtype, "data": "synthetic",
           "config": {"workload": f"{wl.name} swept over B in {Bs} x k in {ks}", "Hq": wl.Hq, "Hkv": wl.Hkv,
                      "D": wl.D, "V": wl.V, "sigma": wl.sigma, "kv_len": f"{wl.len_dist}[{wl.len_lo},{wl.len_hi}]"},
           "sweep": rows,
           "solver": {"note": "respec_solver_pick on this sweep; step time MODELLED as layers x attention + sampler, "
                              "one drafter step = draft_cost_ratio x the plain decoding step",
                      "table": solver_table(rows) if any(r["k"] == 0 for r in rows) else None}}
    print(json.dumps(out))


def run_copy_probe(mib: int, iters: int):
    """A plain device-to-device copy of known size, for calibrating rocprofv3's byte counters: what
    FETCH_SIZE / WRITE_SIZE report for its kernel, divided by the bytes copied, is the factor applied
    to the same counters of the verify kernels."""
    n = mib << 20
    src = torch.arange(n // 4, dtype=torch.int32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(iters):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_probe_bytes": n, "iters": iters}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="qwen7b_b256_k3", choices=sorted(synth.WORKLOADS))
    ap.add_argument("--sigma", type=float, default=None, help="drafter noise (default: workload's)")
    ap.add_argument("--batch", type=int, default=None, help="override B (sweeps)")
    ap.add_argument("--k", type=int, default=None, help="override k (sweeps)")
    ap.add_argument("--tree", default=None, metavar="DEPTHxBRANCH",
                    help="time the tree-of-drafts entry points: a chain of DEPTH nodes, BRANCH candidates per position")
    ap.add_argument("--page-size", type=int, default=None,
                    help="run on a paged KV cache with pages of this many tokens (adds the commit kernel to the step)")
    ap.add_argument("--probe-every", type=int, default=4,
                    help="in the timed region, bracket the main attention kernel with events on every n-th step")
    ap.add_argument("--layers", type=int, default=None,
                    help="attention layers of the modelled full-depth figure (default: the model's public card)")
    ap.add_argument("--measure-depth", action=argparse.BooleanOptionalAction, default=None,
                    help="also time the step with one attention call per layer, each layer on a KV cache of its "
                         "own (default: on when those caches take less than 64 GB; never in --sweep)")
    ap.add_argument("--rotate", type=int, default=1,
                    help="copies of the KV cache and the logits used in turn (cold-cache timing of small workloads)")
    ap.add_argument("--cpu-seqs", type=int, default=256,
                    help="sequences the oracle is timed on (cpu_baseline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep", action="store_true",
                    help="time the verify step over --sweep-batches x --sweep-ks of the workload (k = 0: plain decoding)")
    ap.add_argument("--sweep-batches", default="64,256,512,1024")
    ap.add_argument("--sweep-ks", default="0,1,2,4,8")
    ap.add_argument("--kd-rows", type=int, default=None,
                    help="time respec_kd_rows on this many row pairs instead of the verify step")
    ap.add_argument("--copy-probe", type=int, default=None, metavar="MIB",
                    help="only copy this many MiB device to device three times (calibrates rocprofv3's byte counters)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the verify step shards over sequences with "
              "no exchange, so --gpus N > 1 is not measured here", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)

    import dataclasses
    wl = synth.WORKLOADS[args.workload]
    changes = {}
    if args.sigma is not None:
        changes["sigma"] = args.sigma
    if args.batch is not None:
        changes["B"] = args.batch
    if args.k is not None:
        changes["k"] = args.k
    if changes:
        wl = dataclasses.replace(wl, **changes)

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    if args.copy_probe:
        run_copy_probe(args.copy_probe, 3)
        return
    if args.kd_rows:
        run_kd(args, wl, dev)
        return
    if args.sweep:
        run_sweep(args, wl, dev)
        return
    line = bench_verify(args, wl, dev, bool(changes), not args.no_cpu_baseline)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
