"""GPU parity of respec_rejection_sample against the CPU oracle.

Tokens and accepted counts must match bit-exactly given the same uniforms; the only
exceptions allowed are sequences the oracle flags as boundary draws (an acceptance test
within 1e-6 of the ratio, or u*Z within 1e-6*Z of a CDF edge), which are counted.
"""
import numpy as np
import pytest
import torch
from scipy import stats

from helpers import compare_sampler, env_setting, flag_bound, gpu_sample, oracle_sample, sampler_split
from paper_2510_26475_amd import binding, synth

pytestmark = pytest.mark.gpu


def _wl(name, V, dtype, sigma=1.0, T=1.0):
    return synth.Workload(name, B=0, k=0, Hq=1, Hkv=1, D=64, V=V, dtype=dtype,
                          len_dist="uniform", len_lo=1, len_hi=1, sigma=sigma, temperature=T)


def _batch(wl, ks, seed):
    return synth.make_batch(wl, device="cuda", kv_lens=[k + 1 for k in ks], k_per_seq=ks,
                            seed=seed, with_attention=False)


def _parity(oracle, batch, **kw):
    gpu = gpu_sample(batch, **kw)
    ref = oracle_sample(oracle, batch, **kw)
    tally = compare_sampler(gpu, ref)
    # boundary draws: no more than the recipe's logits make likely (mean + 4 sd, see flag_bound)
    assert tally["flagged"] <= flag_bound(tally["B"], batch.wl.V), tally
    print(f"{batch.wl.name}: B={tally['B']} flagged by the oracle {tally['flagged']}, by the GPU "
          f"{tally['gpu_flagged']}, flagged sequences that differ {tally['flagged_mismatch']}")
    return gpu, ref, tally


def test_tiny_f32_workload(oracle):
    wl = synth.WORKLOADS["tiny_f32"]
    batch = synth.make_batch(wl, device="cuda", with_attention=False)
    gpu, ref, _ = _parity(oracle, batch)
    assert (ref[1] >= 0).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V", [1024, 1000, 1001, 7, 4099])
def test_small_vocab_sizes_and_ragged_tails(oracle, dtype, V):
    # V = 1001 / 7 / 4099: rows are not 16-byte aligned and end in a partial slot
    wl = _wl("small", V, dtype)
    ks = [4, 0, 3, 1, 4, 2, 4, 4] * 8
    _, ref, _ = _parity(oracle, _batch(wl, ks, seed=V))
    assert len(set(ref[1].tolist())) >= 3          # a mix of acceptance lengths


@pytest.mark.parametrize("sigma", [0.5, 1.0, 2.0])
def test_full_vocab_bf16(oracle, sigma):
    wl = _wl("full_bf16", 151936, "bf16", sigma=sigma)
    gpu, ref, tally = _parity(oracle, _batch(wl, [3] * 24 + [4] * 8, seed=int(10 * sigma)))
    # a flagged draw sits within 1e-6 (relative) of a decision boundary and the HIP path's sums
    # carry a few 1e-7: at most about half of the flagged draws may come out on the other side
    assert tally["flagged_mismatch"] <= max(1, (tally["flagged"] + 1) // 2), tally


def test_full_vocab_f32_with_temperature(oracle):
    wl = _wl("full_f32", 151936, "f32", sigma=1.0, T=0.6)
    _parity(oracle, _batch(wl, [3] * 12, seed=77))


def test_ragged_draft_lengths_full_vocab(oracle):
    wl = _wl("ragged", 151936, "bf16", sigma=1.0)
    ks = [0, 8, 3, 1, 7, 0, 5, 2, 8, 4, 6, 0]
    gpu, ref, _ = _parity(oracle, _batch(wl, ks, seed=5))
    for b, k in enumerate(ks):
        assert (gpu[0][b, gpu[1][b] + 1:] == -1).all() and gpu[1][b] <= k


def test_identical_drafter_accepts_everything(oracle):
    wl = _wl("same", 151936, "bf16")
    ks = [4, 2, 0, 3]
    batch = _batch(wl, ks, seed=6)
    qi = batch.q_indptr.tolist()
    for b, k in enumerate(ks):                     # drafter rows become byte copies of the target's
        batch.draft_logits[qi[b] - b: qi[b] - b + k] = batch.target_logits[qi[b]: qi[b] + k]
    batch.u_accept.fill_(float(np.float32(1.0) - np.float32(2.0 ** -24)))
    gpu, ref, _ = _parity(oracle, batch)
    assert gpu[1].tolist() == ks


@pytest.mark.parametrize("env", ["RESPEC_SAMPLER_GUARDED", "RESPEC_SAMPLER_TWO_TERM", "RESPEC_SAMPLER_NO_TABLE"])
def test_alternative_normaliser_passes_agree(oracle, env, monkeypatch):
    # the guarded pass (running per-thread references) and the two-term exponent are the paths
    # taken for unaligned rows / temperatures whose log2(e)/T rounds badly; without the table of
    # slot totals the final draw reads its region again (rows too wide for LDS); force them here
    monkeypatch.setenv(env, "1")
    wl = _wl("alt", 151936, "bf16", sigma=1.0)
    _parity(oracle, _batch(wl, [3] * 16 + [0, 1, 2, 4], seed=21))


def test_f32_logits_full_vocab_are_too_wide_for_the_slot_table(oracle):
    # 151,936 f32 logits are 37,984 slots (148 KB of totals): the draw falls back to re-reading
    _parity(oracle, _batch(_wl("wide_f32", 151936, "f32", sigma=1.0), [3] * 12 + [0, 2], seed=22))


@pytest.mark.parametrize("V", [24576 * 8, 24576 * 8 + 8])
def test_rows_at_the_edge_of_the_slot_table(oracle, V):
    # 24,576 slots are exactly the 96 KB the table may take; one more slot goes without it
    _parity(oracle, _batch(_wl("edge", V, "bf16", sigma=1.0), [2] * 10 + [0, 3], seed=23))


def test_huge_outlier_logit_takes_the_guarded_pass(oracle):
    # one logit far above a wave's first slots overflows the fast pass, which must then be
    # repeated with the guarded one; -inf runs at the row start leave a wave without reference
    wl = _wl("outlier", 151936, "bf16", sigma=1.0)
    batch = _batch(wl, [2] * 8, seed=22)
    batch.target_logits[0, 100000] = 400.0
    batch.draft_logits[1, 77] = 300.0
    batch.target_logits[3, :40000] = float("-inf")
    batch.draft_logits[2, :40000] = float("-inf")
    batch.target_logits[5, 5] = 250.0
    batch.draft_logits[4, 5] = 250.0
    gpu, ref, _ = _parity(oracle, batch)


def test_bonus_rows_drawn_in_one_pass_and_their_fallbacks(oracle):
    # the bonus token (and plain sampling, k = 0) is drawn in one pass against a reference taken
    # from the row's first 512 slots; a logit far above it overflows that pass and a row start
    # without finite logits gives no reference: both fall back to normaliser pass plus draw
    wl = _wl("bonus", 151936, "bf16", sigma=1.0)
    ks = [0] * 10 + [2, 3]
    batch = _batch(wl, ks, seed=41)
    qi = batch.q_indptr.tolist()
    batch.target_logits[qi[0], 100000] = 400.0          # overflows the one-pass weights
    batch.target_logits[qi[1], :5000] = float("-inf")   # no reference in the first 512 slots
    batch.target_logits[qi[2], 140001] = 60.0           # far above the reference, still in range
    batch.target_logits[qi[3], 17] = 90.0               # the reference itself is the outlier
    batch.target_logits[qi[4], 4096:] = float("-inf")   # all the mass inside the first 512 slots
    for b in (10, 11):                                   # every draft accepted: the bonus row is used
        k = ks[b]
        batch.draft_logits[qi[b] - b: qi[b] - b + k] = batch.target_logits[qi[b]: qi[b] + k]
    batch.u_accept.fill_(0.25)
    ref = oracle_sample(oracle, batch)
    for workspace in (None, "shared"):   # one work-group per sequence (the one-pass form), and shared
        gpu = gpu_sample(batch, workspace=workspace)
        tally = compare_sampler(gpu, ref)
        assert tally["flagged"] <= 2, tally
        assert gpu[1].tolist() == ks
        assert gpu[0][0, 0] == 100000 and gpu[0][3, 0] == 17


@pytest.mark.parametrize("split", [1, 2, 4, 8])
def test_sequences_shared_by_several_work_groups(oracle, split):
    # the vocabulary of a sequence is cut into `split` parts that exchange partial sums; the
    # mailbox workspace is reused from call to call without being cleared
    wl = _wl("shared", 151936, "bf16", sigma=1.0)
    ks = [3, 0, 4, 1, 2, 4, 3, 3, 0, 2, 4, 1]
    batch = _batch(wl, ks, seed=31)
    ref = oracle_sample(oracle, batch)
    with sampler_split(split):
        for _ in range(3):
            gpu = gpu_sample(batch)
            tally = compare_sampler(gpu, ref)
            assert tally["flagged"] <= 3, tally


@pytest.mark.parametrize("two_items", [0, 1])
@pytest.mark.parametrize("split", [2, 4, 8])
def test_shared_sequences_one_or_two_chain_items_per_stage(oracle, split, two_items):
    # a shared sequence may take the normalisers of two consecutive items of its chain (two
    # positions, or the last position and the bonus token's row) in one exchange; both ways must
    # give the oracle's tokens, for every chain length and for chains that end at every position
    wl = _wl("two_items", 151936, "bf16", sigma=0.5)
    ks = [4] * 12 + [3, 0, 1, 2, 3, 4, 2, 1]
    batch = _batch(wl, ks, seed=37)
    ref = oracle_sample(oracle, batch)
    n_acc = ref[1].tolist()
    assert len(set(n_acc)) >= 3 and 4 in n_acc     # rejections at several positions and full chains
    with sampler_split(split), env_setting("RESPEC_SAMPLER_TWO_ITEMS", two_items):
        for _ in range(2):
            tally = compare_sampler(gpu_sample(batch), ref)
            assert tally["flagged"] <= 4, tally


@pytest.mark.parametrize("dtype,T", [("f32", 0.7), ("bf16", 0.6), ("f32", 1.0)])
def test_two_chain_items_per_stage_in_the_other_kernel_forms(oracle, dtype, T):
    # f32 logits and temperatures whose exponent constant takes the two-term form: the other
    # instantiations of the shared kernel
    wl = _wl("two_items_forms", 50000, dtype, sigma=0.5, T=T)
    ks = [4] * 6 + [3, 0, 1, 2]
    batch = _batch(wl, ks, seed=43)
    ref = oracle_sample(oracle, batch)
    for two_items in (0, 1):
        with sampler_split(4), env_setting("RESPEC_SAMPLER_TWO_ITEMS", two_items):
            tally = compare_sampler(gpu_sample(batch), ref)
            assert tally["flagged"] <= 3, tally


@pytest.mark.parametrize("two_items", [0, 1])
def test_shared_sequences_never_use_rows_past_the_first_rejection(oracle, two_items):
    # with two items per stage the row pair after a rejected position is read ahead of the test
    # that makes it unnecessary; whatever it holds (here NaN) must not reach the outputs
    wl = _wl("poison_shared", 151936, "bf16", sigma=1.5)
    ks = [4] * 12
    batch = _batch(wl, ks, seed=9)
    ref = oracle_sample(oracle, batch)
    qi = batch.q_indptr.tolist()
    for b, k in enumerate(ks):
        n = int(ref[1][b])
        batch.target_logits[qi[b] + n + 1: qi[b + 1]] = float("nan")
        d0 = qi[b] - b
        batch.draft_logits[d0 + n + 1: d0 + k] = float("nan")
        batch.u_accept[d0 + n + 1: d0 + k] = float("nan")
    with sampler_split(4), env_setting("RESPEC_SAMPLER_TWO_ITEMS", two_items):
        compare_sampler(gpu_sample(batch), ref)
    assert len(set(ref[1].tolist())) >= 3


def test_shared_sequences_with_outliers_repeat_the_item_with_the_guarded_pass(oracle):
    # an overflowing fast pass in one part of one item of a two-item stage: that item alone is
    # repeated by all parts with the guarded pass, the other item's numbers stand
    wl = _wl("outlier_shared", 151936, "bf16", sigma=0.5)
    batch = _batch(wl, [4] * 6, seed=22)
    qi = batch.q_indptr.tolist()
    batch.target_logits[qi[0] + 1, 100000] = 400.0     # second item of sequence 0's first stage
    batch.draft_logits[qi[1] - 1 + 0, 77] = 300.0       # first item of sequence 1's first stage
    batch.target_logits[qi[2] + 4, 5] = 350.0           # the bonus row of sequence 2
    batch.target_logits[qi[3] + 2, :60000] = float("-inf")
    ref = oracle_sample(oracle, batch)
    for split in (2, 8):
        with sampler_split(split), env_setting("RESPEC_SAMPLER_TWO_ITEMS", 1):
            compare_sampler(gpu_sample(batch), ref)


@pytest.mark.parametrize("V", [1000, 70, 4099])
def test_shared_sequences_with_small_and_ragged_vocabularies(oracle, V):
    # parts without any slot, unaligned rows, a partial last slot
    wl = _wl("shared_small", V, "bf16")
    ks = [2, 0, 3, 1] * 4
    batch = _batch(wl, ks, seed=V + 1)
    ref = oracle_sample(oracle, batch)
    for split in (2, 8):
        with sampler_split(split):
            compare_sampler(gpu_sample(batch), ref)


def test_a_mailbox_marked_unusable_reports_failure_until_it_is_zeroed(oracle):
    """What a call whose wait ran out leaves behind, forced from the host: the epoch word of one
    sequence's mailbox holds the poison value.  Every work-group of that sequence then reports
    failure at once (no waiting), the other sequences are untouched, and a zeroed workspace works
    again."""
    wl = _wl("poisoned_box", 151936, "bf16")
    ks = [3, 1, 0, 2, 3, 3]
    batch = _batch(wl, ks, seed=41)
    ref = oracle_sample(oracle, batch)
    B, V = len(ks), 151936
    ws = torch.zeros(binding.respec_rejection_sample_workspace_bytes(B, B, V, binding.RESPEC_BF16),
                     dtype=torch.uint8, device="cuda")
    box = ws.numel() // B
    with sampler_split(4):
        compare_sampler(gpu_sample(batch, workspace=ws), ref)            # a healthy call first
        ws.view(torch.int32)[2 * box // 4] = -1                            # sequence 2's epoch word = 0xffffffff
        toks, n, flags = gpu_sample(batch, workspace=ws)
        assert n[2] == -1
        keep = [b for b in range(B) if b != 2]
        compare_sampler((toks[keep], n[keep], flags[keep]), tuple(r[keep] for r in ref))
        toks, n, flags = gpu_sample(batch, workspace=ws)                   # it stays that way
        assert n[2] == -1
        ws.zero_()
        compare_sampler(gpu_sample(batch, workspace=ws), ref)


def test_a_forced_split_never_outgrows_the_device(oracle):
    """All parts of a sequence wait for one another, so the library launches no more work-groups
    than the device has compute units: a forced split of 8 on 96 sequences is cut down and the
    results are what they always are."""
    wl = _wl("clamped_split", 32768, "bf16")
    batch = _batch(wl, [2, 3, 1, 0] * 24, seed=43)
    ref = oracle_sample(oracle, batch)
    with sampler_split(8):
        compare_sampler(gpu_sample(batch), ref)


def test_without_a_workspace_one_work_group_walks_a_sequence(oracle):
    wl = _wl("nows", 151936, "bf16")
    batch = _batch(wl, [3, 1, 0, 2], seed=33)
    compare_sampler(gpu_sample(batch, workspace=None), oracle_sample(oracle, batch))


def test_no_drafts_at_all_is_plain_sampling(oracle):
    wl = _wl("k0", 32000, "bf16")
    gpu, ref, _ = _parity(oracle, _batch(wl, [0] * 64, seed=7))
    assert (gpu[1] == 0).all() and gpu[0].shape == (64, 1)


def test_disjoint_supports_and_masked_vocab(oracle):
    wl = _wl("disjoint", 4096, "f32")
    batch = _batch(wl, [1] * 32, seed=8)
    batch.target_logits[:, 1::2] = float("-inf")
    batch.draft_logits[:, 0::2] = float("-inf")
    batch.draft_tokens[:] = 2 * torch.randint(0, 2048, (32,), device="cuda", dtype=torch.int32) + 1
    batch.u_accept.fill_(0.5)
    gpu, ref, _ = _parity(oracle, batch)
    assert (gpu[1] == 0).all() and (gpu[0][:, 0] % 2 == 0).all()


def test_rows_after_the_first_rejection_are_never_read(oracle):
    wl = _wl("poison", 151936, "bf16", sigma=1.5)
    ks = [4] * 16
    batch = _batch(wl, ks, seed=9)
    base = gpu_sample(batch)
    qi = batch.q_indptr.tolist()
    for b, k in enumerate(ks):
        n = int(base[1][b])
        batch.target_logits[qi[b] + n + 1: qi[b + 1]] = float("nan")
        d0 = qi[b] - b
        batch.draft_logits[d0 + n + 1: d0 + k] = float("nan")
        batch.u_accept[d0 + n + 1: d0 + k] = float("nan")
    again = gpu_sample(batch)
    for a, c in zip(base, again):
        np.testing.assert_array_equal(a, c)
    assert len(set(base[1].tolist())) >= 3


def test_runs_are_bitwise_reproducible(oracle):
    wl = _wl("det", 151936, "bf16")
    batch = _batch(wl, [3] * 32, seed=10)
    a, b = gpu_sample(batch), gpu_sample(batch)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x, y)


def test_chi_square_emitted_marginal_is_target_on_gpu(oracle):
    """Losslessness (Section 2.2): 10^6 sequences, k = 1, tiny vocabulary, all on the GPU path."""
    V, N = 12, 1_000_000
    g = torch.Generator(device="cpu").manual_seed(3)
    t_row = 1.5 * torch.randn(V, generator=g)
    d_row = t_row + torch.randn(V, generator=g)
    wl = _wl("chi", V, "f32")
    target = t_row.repeat(2 * N, 1).cuda()
    draft = d_row.repeat(N, 1).cuda()
    dg = torch.Generator(device="cuda").manual_seed(4)
    toks_in = synth.sample_draft_tokens(draft, 1.0, dg, chunk_rows=1 << 18)
    batch = synth.VerifyBatch(
        wl=wl, q=torch.empty(0), k_cache=torch.empty(0), v_cache=torch.empty(0),
        q_indptr=torch.arange(0, 2 * N + 1, 2, dtype=torch.int32, device="cuda"),
        kv_indptr=torch.empty(0), target_logits=target, draft_logits=draft, draft_tokens=toks_in,
        u_accept=torch.rand(N, generator=dg, device="cuda"),
        u_final=torch.rand(N, generator=dg, device="cuda"), k_per_seq=[1] * N, kv_lens=[2] * N)
    toks, n, _ = gpu_sample(batch)
    p = oracle.softmax_rows(t_row.numpy()[None].astype(np.float32), 1.0, oracle.F32)[0]
    q = oracle.softmax_rows(d_row.numpy()[None].astype(np.float32), 1.0, oracle.F32)[0]
    counts = np.bincount(toks[:, 0], minlength=V)
    assert stats.chisquare(counts, p * N)[1] > 1e-3
    alpha = np.minimum(p, q).sum()
    assert abs(n.mean() - alpha) < 4.0 * np.sqrt(alpha * (1 - alpha) / N)


def test_qwen7b_headline_workload_full_batch(oracle):
    """B=256, k=3, V=151936 bf16 in the launch configuration the benchmark times; the oracle
    walks the whole batch."""
    wl = synth.WORKLOADS["qwen7b_b256_k3"]
    batch = synth.make_batch(wl, device="cuda", with_attention=False)
    gpu, ref, tally = _parity(oracle, batch)
    emitted = float((ref[1] + 1).mean())
    assert 1.8 < emitted < 2.8, emitted           # closed form at sigma = 1, k = 3 is about 2.27
    print("qwen7b sampler tally", tally, "emitted/seq", emitted)


@pytest.mark.parametrize("B", [64, 16])
def test_qwen3b_small_batches_in_the_library_s_own_choice_of_sharing(oracle, B):
    """B = 64 (the baseline's small workload) and B = 16, k = 4, V = 151936 bf16 with the mailbox
    workspace and no knob set: the library shares a sequence among four or eight work-groups and
    takes two chain items per exchange; three calls in a row on one workspace."""
    import dataclasses
    wl = dataclasses.replace(synth.WORKLOADS["qwen3b_b64_k4"], B=B)
    batch = synth.make_batch(wl, device="cuda", with_attention=False)
    ref = oracle_sample(oracle, batch)
    from helpers import sampler_workspace
    ws = sampler_workspace(B, wl.V, binding.RESPEC_BF16, "cuda")
    for _ in range(3):
        tally = compare_sampler(gpu_sample(batch, workspace=ws), ref)
        assert tally["flagged"] <= flag_bound(B, wl.V), tally
    assert len(set(ref[1].tolist())) >= 4      # chains of every length, full ones among them


def test_bad_arguments_are_rejected_before_any_launch():
    wl = _wl("err", 1024, "f32")
    batch = _batch(wl, [2, 2], seed=1)
    toks = torch.empty((2, 3), dtype=torch.int32, device="cuda")
    n = torch.empty(2, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.RespecError) as e:
        binding.respec_rejection_sample(batch.target_logits, batch.draft_logits,
                                        batch.draft_tokens, batch.q_indptr, batch.u_accept,
                                        batch.u_final, toks, n, None, 2, 0.0)
    assert e.value.status == 1
    with pytest.raises(binding.RespecError):
        binding.respec_rejection_sample(batch.target_logits, batch.draft_logits,
                                        batch.draft_tokens, batch.q_indptr, batch.u_accept,
                                        batch.u_final, toks[:, :2].contiguous(), n, None, 1, 1.0)


@pytest.mark.parametrize("no_table", [0, 1])
def test_extreme_final_uniforms_pick_tokens_with_mass(oracle, no_table, monkeypatch):
    """u_final = 0 and the largest binary32 below 1 sit on a CDF edge by construction (always
    flagged, so parity says nothing): the token drawn must still carry mass, the first such
    token for u = 0 and one at the far end of the support for u -> 1."""
    if no_table:
        monkeypatch.setenv("RESPEC_SAMPLER_NO_TABLE", "1")
    wl = _wl("extreme", 151936, "bf16", sigma=1.0)
    ks = [2] * 16 + [0] * 4
    batch = _batch(wl, ks, seed=31)
    B = len(ks)
    u = np.zeros(B, dtype=np.float32)
    u[1::2] = np.float32(1.0) - np.float32(2.0 ** -24)
    batch.u_final.copy_(torch.from_numpy(u))
    toks, n, _ = gpu_sample(batch, workspace=None)
    ref_t, ref_n, ref_f = oracle_sample(oracle, batch)
    assert np.array_equal(n, ref_n)                      # the acceptance tests do not involve u_final
    P = oracle.softmax_rows(synth.to_host_array(batch.target_logits), 1.0, oracle.BF16)
    Q = oracle.softmax_rows(synth.to_host_array(batch.draft_logits), 1.0, oracle.BF16)
    qi = batch.q_indptr.cpu().numpy()
    for b in range(B):
        row = qi[b] + n[b]
        w = P[row] if n[b] == ks[b] else np.maximum(P[row] - Q[qi[b] - b + n[b]], 0.0)
        tok = toks[b, n[b]]
        assert w[tok] > 0.0, (b, tok)
        cdf = np.cumsum(w) / w.sum()
        if u[b] == 0:
            assert cdf[tok] - w[tok] / w.sum() <= 2e-6      # nothing but rounding noise before it
        else:
            assert cdf[tok] >= 1.0 - 2e-6                   # at the far end of the support


@pytest.mark.parametrize("T", [0.25, 0.5, 0.6, 0.7, 1.3, 2.0])
def test_temperatures_on_both_sides_of_the_one_term_criterion(oracle, T):
    """log2(e)/T rounds well for some temperatures (powers of two times 1, a few others) and
    badly for the rest: the former take the one-fma exponent and the fp32 weights of the final
    draw, the latter the two-term exponent and fp64 weights.  Both must agree with the oracle."""
    wl = _wl("temps", 151936, "bf16", sigma=1.0, T=T)
    _, ref, _ = _parity(oracle, _batch(wl, [3] * 20 + [0, 1, 2, 4], seed=int(100 * T)))
    assert len(set(ref[1].tolist())) >= 2
