"""GPU parity of respec_rejection_sample_per_seq (one temperature per sequence, 0 = greedy
verification) against the CPU oracle.

Greedy sequences are integer work (comparisons of stored logits): tokens and counts must match
bit for bit, no exceptions.  Sampled sequences follow the rule of respec_rejection_sample: exact
on sequences the oracle does not flag as boundary draws.
"""
import numpy as np
import pytest
import torch

from helpers import compare_sampler
from paper_2510_26475_amd import binding, synth

pytestmark = pytest.mark.gpu


def _wl(name, V, dtype, sigma=1.0):
    return synth.Workload(name, B=0, k=0, Hq=1, Hkv=1, D=64, V=V, dtype=dtype,
                          len_dist="uniform", len_lo=1, len_hi=1, sigma=sigma, temperature=1.0)


def _batch(wl, ks, seed):
    return synth.make_batch(wl, device="cuda", kv_lens=[k + 1 for k in ks], k_per_seq=ks,
                            seed=seed, with_attention=False)


def _real(t):
    a = synth.to_host_array(t)
    return a if a.dtype == np.float32 else (a.astype(np.uint32) << 16).view(np.float32)


def _draft_the_argmax(batch, temps, prob, seed):
    """Greedy sequences draft the first argmax of their target row with probability `prob`
    (computed on the host with numpy), so that acceptance lengths mix."""
    rng = np.random.default_rng(seed)
    real = _real(batch.target_logits)
    toks = batch.draft_tokens.cpu().numpy().copy()
    qi = batch.q_indptr.tolist()
    for b, k in enumerate(batch.k_per_seq):
        if temps[b] == 0:
            for i in range(k):
                if rng.random() < prob:
                    toks[qi[b] - b + i] = int(np.argmax(real[qi[b] + i]))
    batch.draft_tokens.copy_(torch.from_numpy(toks))


def _gpu(batch, temps, with_drafter=True, max_k=None):
    B = len(batch.k_per_seq)
    max_k = batch.max_k if max_k is None else max_k
    dev = batch.target_logits.device
    toks = torch.full((B, max_k + 1), -7, dtype=torch.int32, device=dev)
    n = torch.full((B,), -7, dtype=torch.int32, device=dev)
    flags = torch.full((B,), -7, dtype=torch.int32, device=dev)
    t = torch.tensor(np.asarray(temps, dtype=np.float32), device=dev)
    binding.respec_rejection_sample_per_seq(
        batch.target_logits, batch.draft_logits if with_drafter else None, batch.draft_tokens, batch.q_indptr,
        batch.u_accept if with_drafter else None, batch.u_final, t, toks, n, flags, max_k)
    torch.cuda.synchronize()
    return toks.cpu().numpy(), n.cpu().numpy(), flags.cpu().numpy()


def _ref(oracle, batch, temps, max_k=None):
    dt = oracle.F32 if batch.wl.dtype == "f32" else oracle.BF16
    n_draft = batch.total_q - len(batch.k_per_seq)
    return oracle.rejection_sample_per_seq(
        synth.to_host_array(batch.target_logits), synth.to_host_array(batch.draft_logits) if n_draft else None,
        batch.draft_tokens.cpu().numpy() if n_draft else None, batch.q_indptr.cpu().numpy(),
        batch.u_accept.cpu().numpy() if n_draft else None, batch.u_final.cpu().numpy(),
        batch.max_k if max_k is None else max_k, np.asarray(temps, dtype=np.float32), dt, n_threads=0)


def _exact(gpu, ref):
    assert np.array_equal(gpu[1], ref[1]), (gpu[1].tolist(), ref[1].tolist())
    assert np.array_equal(gpu[0], ref[0])
    assert not gpu[2].any()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V", [1024, 1001, 7, 4099, 20000])
def test_greedy_small_vocabularies_and_ragged_tails(oracle, dtype, V):
    ks = [4, 0, 3, 1, 4, 2, 4, 4] * 6
    batch = _batch(_wl("g", V, dtype), ks, seed=V)
    temps = [0.0] * len(ks)
    _draft_the_argmax(batch, temps, 0.75, seed=V)
    gpu, ref = _gpu(batch, temps), _ref(oracle, batch, temps)
    _exact(gpu, ref)
    assert len(set(ref[1].tolist())) >= 3


def test_greedy_ties_take_the_lowest_token_id(oracle):
    # logits quantised to a handful of values: every row has many equal maxima
    ks = [3, 2, 0, 3] * 4
    batch = _batch(_wl("ties", 5000, "bf16"), ks, seed=1)
    batch.target_logits.copy_(torch.round(batch.target_logits.float().clamp(-2, 2)).to(torch.bfloat16))
    temps = [0.0] * len(ks)
    _draft_the_argmax(batch, temps, 0.6, seed=2)
    real = _real(batch.target_logits)
    assert ((real == real.max(axis=1, keepdims=True)).sum(axis=1) > 1).all()
    _exact(_gpu(batch, temps), _ref(oracle, batch, temps))


def test_greedy_full_vocab_bf16_without_drafter_data(oracle):
    ks = [3] * 40 + [0, 8, 5, 1]
    batch = _batch(_wl("gfull", 151936, "bf16"), ks, seed=3)
    temps = [0.0] * len(ks)
    _draft_the_argmax(batch, temps, 0.8, seed=4)
    ref = _ref(oracle, batch, temps)
    _exact(_gpu(batch, temps, with_drafter=False), ref)        # no drafter logits, no uniforms
    _exact(_gpu(batch, temps, with_drafter=True), ref)
    assert 0 < ref[1].sum() < sum(ks)


def test_greedy_reads_no_row_after_the_first_rejection(oracle):
    ks = [4] * 8
    batch = _batch(_wl("poison", 151936, "bf16"), ks, seed=5)
    temps = [0.0] * len(ks)
    _draft_the_argmax(batch, temps, 1.0, seed=6)
    toks = batch.draft_tokens.cpu().numpy().copy()
    qi = batch.q_indptr.tolist()
    for b in range(len(ks)):                 # sequence b is rejected at position b % 4
        i = b % 4
        toks[qi[b] - b + i] = (toks[qi[b] - b + i] + 1) % 151936
        batch.target_logits[qi[b] + i + 1: qi[b + 1]] = float("nan")
    batch.draft_tokens.copy_(torch.from_numpy(toks))
    batch.draft_logits.fill_(float("nan"))
    batch.u_accept.fill_(float("nan"))
    batch.u_final.fill_(float("nan"))
    gpu = _gpu(batch, temps)
    assert gpu[1].tolist() == [b % 4 for b in range(len(ks))]
    _exact(gpu, _ref(oracle, batch, temps))


@pytest.mark.parametrize("dtype,V", [("f32", 1024), ("bf16", 151936), ("bf16", 1001)])
def test_mixed_temperatures(oracle, dtype, V):
    ks = [3, 0, 2, 3, 1, 3, 4, 4, 0, 2, 4, 1] * 3
    temps = ([0.6, 0.0, 1.0, 0.0, 0.4, 0.6, 1.0, 0.0, 0.0, 1.5, 0.6, 1.0] * 3)
    batch = _batch(_wl("mixed", V, dtype), ks, seed=7 + V % 5)
    _draft_the_argmax(batch, temps, 0.6, seed=8)
    gpu, ref = _gpu(batch, temps), _ref(oracle, batch, temps)
    tally = compare_sampler(gpu, ref)
    assert tally["flagged"] <= 6, tally
    greedy = np.array(temps) == 0
    assert np.array_equal(gpu[1][greedy], ref[1][greedy]) and np.array_equal(gpu[0][greedy], ref[0][greedy])
    assert len(set(ref[1][~greedy].tolist())) >= 3


def test_one_temperature_for_all_equals_the_scalar_entry_point_on_unflagged_sequences(oracle):
    from helpers import gpu_sample
    ks = [3] * 32
    batch = _batch(_wl("same_T", 151936, "bf16"), ks, seed=9)
    per_seq = _gpu(batch, [0.6] * len(ks))
    scalar = gpu_sample(batch, temperature=0.6, workspace=None)
    ref = _ref(oracle, batch, [0.6] * len(ks))
    compare_sampler(per_seq, ref)
    compare_sampler(scalar, ref)


def test_bad_device_side_temperatures_are_reported_per_sequence():
    ks = [2, 2, 2, 2]
    batch = _batch(_wl("bad", 1024, "f32"), ks, seed=10)
    toks, n, _ = _gpu(batch, [0.0, -1.0, float("nan"), float("inf")])
    assert n[0] >= 0 and n[1:].tolist() == [-1, -1, -1] and (toks[1:] == -1).all()
    # a sampled sequence with drafts but no drafter data
    toks, n, _ = _gpu(batch, [0.0, 1.0, 0.0, 0.0], with_drafter=False)
    assert n[1] == -1 and (n[[0, 2, 3]] >= 0).all()


def test_host_side_argument_errors():
    batch = _batch(_wl("args", 1024, "f32"), [1, 1], seed=11)
    toks = torch.empty((2, 2), dtype=torch.int32, device="cuda")
    n = torch.empty(2, dtype=torch.int32, device="cuda")
    with pytest.raises(TypeError):
        binding.respec_rejection_sample_per_seq(batch.target_logits, batch.draft_logits, batch.draft_tokens,
                                                batch.q_indptr, batch.u_accept, batch.u_final,
                                                torch.zeros(3, device="cuda"), toks, n, None, 1)
    # drafted tokens present but no token array: refused before any launch
    status = binding.load().respec_rejection_sample_per_seq(
        batch.target_logits.data_ptr(), None, None, batch.q_indptr.data_ptr(), None, batch.u_final.data_ptr(),
        torch.zeros(2, device="cuda").data_ptr(), toks.data_ptr(), n.data_ptr(), None, 2, 4, 1, 1024, 1024,
        1024, binding.RESPEC_F32, None)
    assert status == 1
    status = binding.load().respec_rejection_sample_per_seq(
        batch.target_logits.data_ptr(), None, batch.draft_tokens.data_ptr(), batch.q_indptr.data_ptr(), None,
        batch.u_final.data_ptr(), None, toks.data_ptr(), n.data_ptr(), None, 2, 4, 1, 1024, 1024, 1024,
        binding.RESPEC_F32, None)
    assert status == 1                                      # no temperature array


def test_full_size_greedy_batch(oracle):
    """The 7B-shaped workload, every sequence greedy: the whole batch against the oracle."""
    wl = synth.WORKLOADS["qwen7b_b256_k3"]
    batch = synth.make_batch(wl, device="cuda", with_attention=False)
    temps = [0.0] * wl.B
    _draft_the_argmax(batch, temps, 0.7, seed=12)
    _exact(_gpu(batch, temps, with_drafter=False), _ref(oracle, batch, temps))
