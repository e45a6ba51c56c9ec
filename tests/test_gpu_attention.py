"""GPU parity of respec_verify_attention against the CPU oracle (element by element).

Tolerances are the contract's: max abs error 2e-2 for bf16, 1e-5 for fp32.  bf16 cases also
check a tighter rms bound (the bf16 rounding of the probabilities and of the output keeps
the rms error near 1e-3 for N(0,1) data), so that a systematic slip cannot hide under 2e-2.
"""
import dataclasses
import math

import numpy as np
import pytest
import torch

from helpers import attn_wgs, check_bf16_attention_rows, env_setting, gpu_attention, oracle_attention, sub_batch
from paper_2510_26475_amd import binding, synth

pytestmark = pytest.mark.gpu

BF16_TOL, F32_TOL = 2e-2, 1e-5


def _wl(name, Hq, Hkv, D, dtype, V=8):
    return synth.Workload(name, B=0, k=0, Hq=Hq, Hkv=Hkv, D=D, V=V, dtype=dtype,
                          len_dist="uniform", len_lo=1, len_hi=1)


def _check(out, lse, ref, ref_lse, dtype, rms_bound=2.5e-3):
    got = out.double().cpu().numpy()
    assert np.isfinite(got).all(), "output holds NaN/inf (a row was not written?)"
    err = np.abs(got - ref)
    tol = F32_TOL if dtype == "f32" else BF16_TOL
    assert err.max() <= tol, f"max abs err {err.max():.3e} > {tol}"
    if dtype == "bf16":
        check_bf16_attention_rows(got, ref, rms_bound)
    if lse is not None:
        lerr = np.abs(lse.double().cpu().numpy() - ref_lse)
        assert lerr.max() <= (1e-4 if dtype == "f32" else 2e-2), f"lse err {lerr.max():.3e}"
    return float(err.max())


def _run(oracle, wl, lens, ks, seed=0, wgs=None, sm_scale=None):
    batch = synth.make_batch(wl, device="cuda", kv_lens=lens, k_per_seq=ks, seed=seed,
                             with_logits=False)
    with attn_wgs(wgs):
        out, lse = gpu_attention(batch, sm_scale=sm_scale)
    ref, ref_lse = oracle_attention(oracle, batch, sm_scale=sm_scale)
    return _check(out, lse, ref, ref_lse, wl.dtype), batch, out


def test_tiny_f32_workload(oracle):
    wl = synth.WORKLOADS["tiny_f32"]
    batch = synth.make_batch(wl, device="cuda", with_logits=False)
    out, lse = gpu_attention(batch)
    ref, ref_lse = oracle_attention(oracle, batch)
    _check(out, lse, ref, ref_lse, "f32")


def test_f32_longer_contexts(oracle):
    wl = _wl("f32_long", 4, 2, 64, "f32")
    _run(oracle, wl, [300, 129, 5, 1000, 128, 513], [4, 0, 4, 2, 3, 1], seed=3)
    wl = _wl("f32_long_d128", 6, 2, 128, "f32")
    _run(oracle, wl, [257, 31, 640], [2, 4, 0], seed=4)


@pytest.mark.parametrize("heads", [(28, 4), (16, 2), (40, 8), (4, 1), (8, 8), (7, 1)])
@pytest.mark.parametrize("wgs", [None, 1, 3, 64])
def test_bf16_d128_shapes(oracle, heads, wgs):
    Hq, Hkv = heads
    wl = _wl("bf16_shapes", Hq, Hkv, 128, "bf16")
    lens = [33, 130, 257, 1000, 6, 5, 128, 129, 2049]
    ks = [3, 4, 0, 4, 4, 4, 1, 2, 3]
    _run(oracle, wl, lens, ks, seed=Hq + (wgs or 0), wgs=wgs)


@pytest.mark.parametrize("wgs", [None, 5])
def test_bf16_d64(oracle, wgs):
    wl = _wl("bf16_d64", 8, 2, 64, "bf16")
    _run(oracle, wl, [33, 130, 700, 9, 257], [3, 4, 0, 8, 2], seed=11, wgs=wgs)


@pytest.mark.parametrize("k", [0, 1, 2, 4, 8])
def test_bf16_draft_lengths_14b_heads(oracle, k):
    # G = 5: 5, 10, 15, 25, 45 MFMA columns -> 1..3 column tiles
    wl = _wl("bf16_k", 40, 8, 128, "bf16")
    _run(oracle, wl, [1500, 64 + k, 333], [k, k, k], seed=20 + k, wgs=37)


@pytest.mark.parametrize("quad", [1, 0])
@pytest.mark.parametrize("wgs", [None, 1, 3, 11, 64])
@pytest.mark.parametrize("shape", [(16, 2, 128, 8), (28, 4, 128, 12), (16, 2, 128, 15), (16, 2, 128, 17),
                                   (8, 1, 64, 10), (40, 8, 128, 20), (32, 2, 128, 15)])
def test_more_than_64_columns(oracle, shape, wgs, quad):
    """65 .. 256 MFMA columns (72, 91, 128, 144, 88, 105, 256).  quad = 1: column blocks of 128 with the
    four consumers of a work-group on one range; quad = 0: column blocks of 64."""
    Hq, Hkv, D, k = shape
    wl = _wl("bf16_wide", Hq, Hkv, D, "bf16")
    lens = [400, 90, 1025, 33, 2049, 64 + k, k + 1]
    ks = [k, k, k - 3, k, k, k, k]
    with env_setting("RESPEC_ATTN_QUAD", quad):
        _run(oracle, wl, lens, ks, seed=31 + Hq + k + (wgs or 0), wgs=wgs)


@pytest.mark.parametrize("wgs", [None, 1, 2, 3, 7, 64, 500])
@pytest.mark.parametrize("heads", [(28, 4, 6), (28, 4, 8), (40, 8, 8), (16, 2, 8), (7, 1, 5)])
def test_wide_column_blocks_share_a_range_between_two_consumers(oracle, heads, wgs):
    # 33..72 MFMA columns at D = 128: two consumers per range, each with half of the columns
    Hq, Hkv, k = heads
    wl = _wl("bf16_two_way", Hq, Hkv, 128, "bf16")
    lens = [33, 130, 257, 1000, 9, 10, 128, 129, 2049, 64, 65]
    ks = [k, k, 0, k, k, k - 1, 1, 2, k, k, 3]
    _run(oracle, wl, lens, ks, seed=Hq + k + (wgs or 0), wgs=wgs)


@pytest.mark.parametrize("wgs", [None, 1, 3, 64])
@pytest.mark.parametrize("shape", [(28, 4, 128, 3), (16, 2, 128, 4), (40, 8, 128, 8), (8, 2, 64, 7), (7, 1, 128, 2)])
def test_four_consumers_on_a_block_of_up_to_64_columns(oracle, shape, wgs):
    # 17..64 MFMA columns with the four consumers of a work-group on one range, 16 columns each
    Hq, Hkv, D, k = shape
    wl = _wl("bf16_quad_narrow", Hq, Hkv, D, "bf16")
    lens = [33, 130, 257, 1000, 9, 10, 128, 129, 2049, 64, 65]
    ks = [k, k, 0, k, k, k - 1, 1, 2, k, k, min(3, k)]
    with env_setting("RESPEC_ATTN_QUAD", 2):
        _run(oracle, wl, lens, ks, seed=77 + Hq + k + (wgs or 0), wgs=wgs)


@pytest.mark.parametrize("wide", [0, 1])
@pytest.mark.parametrize("D", [64, 128])
def test_both_forms_of_a_wide_column_block_agree_with_the_oracle(oracle, D, wide):
    wl = _wl("bf16_forms", 40, 8, D, "bf16")            # G = 5, k = 8 -> 45 columns
    with env_setting("RESPEC_ATTN_WIDE", wide):
        _run(oracle, wl, [700, 9, 1300, 12, 4096, 257], [8, 8, 8, 7, 8, 8], seed=50 + D + wide)
        _run(oracle, wl, [700, 9, 1300, 12, 4096, 257], [8, 8, 8, 7, 8, 8], seed=60 + D + wide, wgs=13)


def test_ragged_draft_lengths_in_one_batch(oracle):
    wl = _wl("bf16_ragged", 40, 8, 128, "bf16")
    ks = [0, 8, 3, 1, 7, 0, 5, 2]
    lens = [700, 9, 1300, 2, 4096, 1, 257, 513]
    _run(oracle, wl, lens, ks, seed=41)
    _run(oracle, wl, lens, ks, seed=42, wgs=29)


def test_causal_boundary_with_spiked_keys(oracle):
    """A key with a huge score sits just past each row's horizon: it must capture exactly the
    rows that may see it (2e-2 would not notice an off-by-one on N(0,1) data)."""
    wl = _wl("bf16_spike", 8, 2, 128, "bf16")
    lens, ks = [300, 131, 40, 1029], [4, 3, 4, 2]
    batch = synth.make_batch(wl, device="cuda", kv_lens=lens, k_per_seq=ks, seed=5,
                             with_logits=False)
    qi, ki = batch.q_indptr.tolist(), batch.kv_indptr.tolist()
    G = wl.Hq // wl.Hkv
    for b, (L, k) in enumerate(zip(lens, ks)):
        R = k + 1
        for i in range(R - 1):
            key = L - R + i + 1                      # first key row i must NOT see
            for hk in range(wl.Hkv):
                # aligned with row i (must stay blind to it) and with row i+1 (must be captured)
                qv = batch.q[qi[b] + i, hk * G].float() + batch.q[qi[b] + i + 1, hk * G].float()
                batch.k_cache[ki[b] + key, hk] = (4.0 * qv).to(torch.bfloat16)
                batch.v_cache[ki[b] + key, hk] = 1.5 + 0.125 * i
    for wgs in (None, 2, 13):
        with attn_wgs(wgs):
            out, lse = gpu_attention(batch)
        ref, ref_lse = oracle_attention(oracle, batch)
        _check(out, lse, ref, ref_lse, "bf16", rms_bound=4e-3)
    # the oracle output really is dominated by the spikes (the test has teeth)
    assert (np.abs(ref - 1.5) < 1e-3).mean() > 0.02


def test_cache_holding_only_the_new_tokens(oracle):
    wl = _wl("bf16_min", 28, 4, 128, "bf16")
    err, batch, out = _run(oracle, wl, [4, 1, 5], [3, 0, 4], seed=6)
    # row 0 of a sequence with L = R sees one key: output equals that value row exactly
    v0 = batch.v_cache[0].float().cpu().numpy()          # [Hkv, D]
    got = out[0].float().cpu().numpy().reshape(wl.Hkv, -1, wl.D)
    assert np.array_equal(got, np.broadcast_to(v0[:, None, :], got.shape))


def test_runs_are_bitwise_reproducible(oracle):
    wl = _wl("bf16_det", 28, 4, 128, "bf16")
    batch = synth.make_batch(wl, device="cuda", kv_lens=[3000, 700, 129], k_per_seq=[3, 3, 3],
                             seed=7, with_logits=False)
    with attn_wgs(100):
        a, la = gpu_attention(batch)
        b, lb = gpu_attention(batch)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16)) and torch.equal(la, lb)


def test_rows_beyond_the_batch_are_never_read(oracle):
    wl = _wl("bf16_poison", 16, 2, 128, "bf16")
    lens, ks = [200, 77], [4, 2]
    batch = synth.make_batch(wl, device="cuda", kv_lens=lens, k_per_seq=ks, seed=8,
                             with_logits=False)
    pad = 64
    big_k = torch.full((batch.total_kv + pad, wl.Hkv, wl.D), float("nan"), dtype=torch.bfloat16,
                       device="cuda")
    big_v = big_k.clone()
    big_k[:batch.total_kv] = batch.k_cache
    big_v[:batch.total_kv] = batch.v_cache
    batch.k_cache, batch.v_cache = big_k[:batch.total_kv], big_v[:batch.total_kv]
    out, lse = gpu_attention(batch)
    ref, ref_lse = oracle_attention(oracle, batch)
    _check(out, lse, ref, ref_lse, "bf16")


def test_custom_scale_and_no_lse(oracle):
    wl = _wl("bf16_scale", 8, 2, 128, "bf16")
    batch = synth.make_batch(wl, device="cuda", kv_lens=[500, 64], k_per_seq=[2, 4], seed=9,
                             with_logits=False)
    out, lse = gpu_attention(batch, sm_scale=0.05, want_lse=False)
    assert lse is None
    ref, _ = oracle_attention(oracle, batch, sm_scale=0.05)
    _check(out, None, ref, None, "bf16")


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_a_scale_of_zero_weighs_every_visible_key_alike(oracle, dtype):
    # every score is zero then, hidden keys still count for nothing
    wl = _wl("zero_scale", 8, 2, 128 if dtype == "bf16" else 64, dtype)
    batch = synth.make_batch(wl, device="cuda", kv_lens=[300, 40, 5], k_per_seq=[3, 1, 4], seed=12,
                             with_logits=False)
    out, lse = gpu_attention(batch, sm_scale=0.0)
    ref, ref_lse = oracle_attention(oracle, batch, sm_scale=0.0)
    _check(out, lse, ref, ref_lse, dtype)


def test_qwen3b_workload_full_batch(oracle):
    wl = synth.WORKLOADS["qwen3b_b64_k4"]
    batch = synth.make_batch(wl, device="cuda", with_logits=False)
    out, lse = gpu_attention(batch)
    seqs = sorted(set([int(np.argmax(batch.kv_lens)), int(np.argmin(batch.kv_lens)), 0, 17, 63]))
    sb = sub_batch(batch, seqs)
    ref, ref_lse = oracle_attention(oracle, sb)
    qi = batch.q_indptr.tolist()
    rows = torch.tensor([r for b in seqs for r in range(qi[b], qi[b + 1])], device="cuda")
    _check(out[rows], lse[rows], ref, ref_lse, "bf16")


def test_qwen7b_headline_workload_whole_batch(oracle):
    """Full-size B=256, k=3, 28/4 heads in the launch configuration the benchmark times: every
    row of every sequence against the oracle (which walks the batch in about a second)."""
    wl = synth.WORKLOADS["qwen7b_b256_k3"]
    batch = synth.make_batch(wl, device="cuda", with_logits=False)
    out, lse = gpu_attention(batch)
    ref, ref_lse = oracle_attention(oracle, batch)
    worst = _check(out, lse, ref, ref_lse, "bf16")
    print(f"headline attention: max abs err {worst:.3e} over {batch.total_q} rows")


def test_next_layer_reuses_the_set_up_and_is_bit_equal_to_a_full_call(oracle):
    """The layers of one forward share the index arrays: respec_verify_attention_next_layer skips
    the set-up kernel and must give the bits of a full call on the same arguments."""
    wl = synth.Workload("layers", B=37, k=3, Hq=28, Hkv=4, D=128, V=1024, dtype="bf16",
                        len_dist="uniform", len_lo=40, len_hi=3000, seed=33)
    batch = synth.make_batch(wl, device="cuda", with_logits=False)
    max_q = batch.max_k + 1
    ws = torch.empty(binding.respec_verify_attention_workspace_bytes(
        wl.B, batch.total_q, batch.total_kv, max_q, batch.max_kv_len, wl.Hq, wl.Hkv, wl.D, binding.RESPEC_BF16),
        dtype=torch.uint8, device="cuda")
    g = torch.Generator(device="cuda").manual_seed(5)
    layers = [(batch.q, batch.k_cache, batch.v_cache)]
    for _ in range(2):
        layers.append(tuple(torch.empty_like(t).normal_(generator=g) for t in layers[0]))
    scale = 1.0 / np.sqrt(wl.D)
    full = []
    for q, k, v in layers:
        out = torch.empty_like(q)
        lse = torch.empty((batch.total_q, wl.Hq), dtype=torch.float32, device="cuda")
        binding.respec_verify_attention(q, k, v, batch.q_indptr, batch.kv_indptr, out, lse, max_q,
                                        batch.max_kv_len, scale, ws)
        full.append((out, lse))
    torch.cuda.synchronize()
    # one full call, then the other layers on the same workspace
    ws.zero_()
    outs = []
    for i, (q, k, v) in enumerate(layers):
        out = torch.empty_like(q)
        lse = torch.empty((batch.total_q, wl.Hq), dtype=torch.float32, device="cuda")
        call = binding.respec_verify_attention if i == 0 else binding.respec_verify_attention_next_layer
        call(q, k, v, batch.q_indptr, batch.kv_indptr, out, lse, max_q, batch.max_kv_len, scale, ws)
        outs.append((out, lse))
    torch.cuda.synchronize()
    for (a, la), (b, lb) in zip(full, outs):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)) and torch.equal(la, lb)
    # and the last layer against the oracle
    sb = dataclasses.replace(batch, q=layers[2][0], k_cache=layers[2][1], v_cache=layers[2][2])
    ref, _ = oracle_attention(oracle, sb)
    assert np.abs(outs[2][0].double().cpu().numpy() - ref).max() <= 2e-2


def test_bad_arguments_are_rejected_before_any_launch():
    wl = _wl("bf16_err", 8, 2, 128, "bf16")
    batch = synth.make_batch(wl, device="cuda", kv_lens=[100], k_per_seq=[3], seed=1,
                             with_logits=False)
    out = torch.empty_like(batch.q)
    ws = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.RespecError) as e:       # workspace too small
        binding.respec_verify_attention(batch.q, batch.k_cache, batch.v_cache, batch.q_indptr,
                                        batch.kv_indptr, out, None, 4, 100, 0.1, ws[:16])
    assert e.value.status == 3
    with pytest.raises(binding.RespecError) as e:       # max_q_per_seq too small for total_q
        binding.respec_verify_attention(batch.q, batch.k_cache, batch.v_cache, batch.q_indptr,
                                        batch.kv_indptr, out, None, 2, 100, 0.1, ws)
    assert e.value.status == 1
    q96 = torch.zeros((4, 8, 96), dtype=torch.bfloat16, device="cuda")
    kv96 = torch.zeros((100, 2, 96), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.RespecError) as e:       # head size outside {64,128}
        binding.respec_verify_attention(q96, kv96, kv96, batch.q_indptr, batch.kv_indptr,
                                        torch.empty_like(q96), None, 4, 100, 0.1, ws)
    assert e.value.status == 2
