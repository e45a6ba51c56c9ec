"""Pins for the attention oracle (CPU only).

The oracle is the plain definition of causal grouped-query attention for the k+1 verify
rows of each sequence.  It is pinned here against things that do not come from it: a dense
numpy formulation written independently, closed forms, invariants and a library routine.
"""
import numpy as np
import pytest
import torch

F32, BF16 = 0, 1


def _bf16_bits(x32: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def _bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _as_f64(a, dtype):
    return a.astype(np.float64) if dtype == F32 else _bf16_to_f64(a)


def _indptr(lens):
    out = [0]
    for x in lens:
        out.append(out[-1] + x)
    return np.array(out)


def dense_attention(q, k, v, q_indptr, kv_indptr, Hq, Hkv, sm_scale):
    """Independent dense formulation: full [R, L] score matrix with a -inf mask, einsum."""
    q = np.asarray(q, dtype=np.float64)
    out = np.zeros_like(q)
    lse = np.zeros(q.shape[:2])
    G = Hq // Hkv
    for b in range(len(q_indptr) - 1):
        q0, q1 = q_indptr[b], q_indptr[b + 1]
        s0, s1 = kv_indptr[b], kv_indptr[b + 1]
        R, L = q1 - q0, s1 - s0
        kk = np.repeat(k[s0:s1], G, axis=1)      # [L, Hq, D]
        vv = np.repeat(v[s0:s1], G, axis=1)
        s = sm_scale * np.einsum("rhd,lhd->hrl", q[q0:q1], kk)
        pos_q = (L - R + np.arange(R))[:, None]
        pos_k = np.arange(L)[None, :]
        s = np.where(pos_k <= pos_q, s, -np.inf)
        m = s.max(axis=-1, keepdims=True)
        e = np.exp(s - m)
        den = e.sum(axis=-1, keepdims=True)
        out[q0:q1] = np.einsum("hrl,lhd->rhd", e / den, vv)
        lse[q0:q1] = (m + np.log(den))[..., 0].T
    return out, lse


def _random_case(rng, lens, ks, Hq, Hkv, D, dtype):
    qi, ki = _indptr([k + 1 for k in ks]), _indptr(lens)
    q = rng.standard_normal((qi[-1], Hq, D)).astype(np.float32)
    k = rng.standard_normal((ki[-1], Hkv, D)).astype(np.float32)
    v = rng.standard_normal((ki[-1], Hkv, D)).astype(np.float32)
    if dtype == BF16:
        q, k, v = _bf16_bits(q), _bf16_bits(k), _bf16_bits(v)
    return q, k, v, qi, ki


@pytest.mark.parametrize("dtype", [F32, BF16])
@pytest.mark.parametrize("heads", [(1, 1), (4, 1), (4, 2), (6, 3)])
@pytest.mark.parametrize("D", [4, 64])
def test_matches_dense_brute_force(oracle, dtype, heads, D):
    Hq, Hkv = heads
    rng = np.random.default_rng(100 + D + Hq)
    lens, ks = [17, 5, 9], [4, 4, 0]
    q, k, v, qi, ki = _random_case(rng, lens, ks, Hq, Hkv, D, dtype)
    scale = 1.0 / np.sqrt(D)
    out, lse = oracle.verify_attention(q, k, v, qi, ki, Hq, Hkv, D, scale, dtype, want_lse=True)
    ref, ref_lse = dense_attention(_as_f64(q, dtype), _as_f64(k, dtype), _as_f64(v, dtype),
                                   qi, ki, Hq, Hkv, scale)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, ref_lse, rtol=0, atol=1e-12)


def test_identical_keys_give_running_mean_of_values(oracle):
    rng = np.random.default_rng(1)
    Hq, Hkv, D, L, k = 4, 2, 8, 11, 3
    q, kc, v, qi, ki = _random_case(rng, [L], [k], Hq, Hkv, D, F32)
    kc[:] = kc[0:1]                      # every key equal => uniform attention weights
    out = oracle.verify_attention(q, kc, v, qi, ki, Hq, Hkv, D, 0.3, F32)
    for i in range(k + 1):
        last = L - (k + 1) + i
        mean = v[: last + 1].astype(np.float64).mean(axis=0)     # [Hkv, D]
        for h in range(Hq):
            np.testing.assert_allclose(out[i, h], mean[h // (Hq // Hkv)], atol=1e-13)


def test_constant_values_pass_through(oracle):
    rng = np.random.default_rng(2)
    q, kc, v, qi, ki = _random_case(rng, [9, 6], [2, 1], 4, 1, 16, F32)
    v[:] = 0.0
    v[..., :] = np.linspace(-1, 1, 16, dtype=np.float32)
    out = oracle.verify_attention(q, kc, v, qi, ki, 4, 1, 16, 0.25, F32)
    np.testing.assert_allclose(out, np.broadcast_to(v[0, 0].astype(np.float64), out.shape),
                               atol=1e-13)


def test_cache_of_only_new_tokens_first_row_sees_one_key(oracle):
    rng = np.random.default_rng(3)
    k = 3
    q, kc, v, qi, ki = _random_case(rng, [k + 1], [k], 2, 1, 8, F32)
    out, lse = oracle.verify_attention(q, kc, v, qi, ki, 2, 1, 8, 0.5, F32, want_lse=True)
    for h in range(2):
        np.testing.assert_array_equal(out[0, h], v[0, 0].astype(np.float64))
        s = 0.5 * float(q[0, h].astype(np.float64) @ kc[0, 0].astype(np.float64))
        assert abs(lse[0, h] - s) < 1e-13


def test_causality_future_keys_do_not_matter(oracle):
    rng = np.random.default_rng(4)
    L, k = 12, 3
    q, kc, v, qi, ki = _random_case(rng, [L], [k], 4, 2, 8, F32)
    base = oracle.verify_attention(q, kc, v, qi, ki, 4, 2, 8, 0.35, F32)
    for i in range(k):                       # row k sees everything
        last = L - (k + 1) + i
        k2, v2 = kc.copy(), v.copy()
        k2[last + 1:] = 50.0 * rng.standard_normal(k2[last + 1:].shape)
        v2[last + 1:] = 50.0 * rng.standard_normal(v2[last + 1:].shape)
        pert = oracle.verify_attention(q, k2, v2, qi, ki, 4, 2, 8, 0.35, F32)
        np.testing.assert_array_equal(pert[i], base[i])
        assert np.abs(pert[i + 1] - base[i + 1]).max() > 1e-3     # the next row does see key last+1


def test_key_at_the_boundary_is_visible(oracle):
    # a huge score on the last visible key of row i must capture row i and no earlier row
    rng = np.random.default_rng(5)
    L, k, D = 10, 2, 8
    q, kc, v, qi, ki = _random_case(rng, [L], [k], 1, 1, D, F32)
    i = 1
    last = L - (k + 1) + i
    kc[last, 0] = 100.0 * q[i, 0]
    out = oracle.verify_attention(q, kc, v, qi, ki, 1, 1, D, 1.0, F32)
    np.testing.assert_allclose(out[i, 0], v[last, 0], atol=1e-9)
    assert np.abs(out[i - 1, 0] - v[last, 0]).max() > 1e-2


def test_gqa_heads_with_equal_queries_agree(oracle):
    rng = np.random.default_rng(6)
    Hq, Hkv, D = 6, 2, 8
    q, kc, v, qi, ki = _random_case(rng, [13, 7], [2, 3], Hq, Hkv, D, F32)
    G = Hq // Hkv
    for hk in range(Hkv):
        q[:, hk * G:(hk + 1) * G] = q[:, hk * G:hk * G + 1]
    out = oracle.verify_attention(q, kc, v, qi, ki, Hq, Hkv, D, 0.4, F32)
    for hk in range(Hkv):
        for g in range(1, G):
            np.testing.assert_array_equal(out[:, hk * G + g], out[:, hk * G])
    assert np.abs(out[:, 0] - out[:, G]).max() > 1e-3       # different KV heads differ


def test_batch_permutation(oracle):
    rng = np.random.default_rng(7)
    lens, ks = [9, 14, 6], [1, 3, 0]
    Hq, Hkv, D = 4, 2, 8
    q, kc, v, qi, ki = _random_case(rng, lens, ks, Hq, Hkv, D, F32)
    out = oracle.verify_attention(q, kc, v, qi, ki, Hq, Hkv, D, 0.3, F32)
    perm = [2, 0, 1]
    qp = np.concatenate([q[qi[b]:qi[b + 1]] for b in perm])
    kp = np.concatenate([kc[ki[b]:ki[b + 1]] for b in perm])
    vp = np.concatenate([v[ki[b]:ki[b + 1]] for b in perm])
    outp = oracle.verify_attention(qp, kp, vp, _indptr([ks[b] + 1 for b in perm]),
                                   _indptr([lens[b] for b in perm]), Hq, Hkv, D, 0.3, F32)
    ref = np.concatenate([out[qi[b]:qi[b + 1]] for b in perm])
    np.testing.assert_array_equal(outp, ref)


def test_split_cache_merges_through_log_sum_exp(oracle):
    # attention over a cache cut in two, merged with the (max, sum) rule, equals the whole
    rng = np.random.default_rng(8)
    Hq, Hkv, D, L = 4, 2, 8, 21
    q, kc, v, qi, ki = _random_case(rng, [L], [0], Hq, Hkv, D, F32)
    whole, lse = oracle.verify_attention(q, kc, v, qi, ki, Hq, Hkv, D, 0.3, F32, want_lse=True)
    for cut in (1, 8, 20):
        o1, l1 = oracle.verify_attention(q, kc[:cut], v[:cut], qi, _indptr([cut]), Hq, Hkv, D,
                                         0.3, F32, want_lse=True)
        o2, l2 = oracle.verify_attention(q, kc[cut:], v[cut:], qi, _indptr([L - cut]), Hq, Hkv,
                                         D, 0.3, F32, want_lse=True)
        m = np.maximum(l1, l2)
        w1, w2 = np.exp(l1 - m), np.exp(l2 - m)
        merged = (w1[..., None] * o1 + w2[..., None] * o2) / (w1 + w2)[..., None]
        np.testing.assert_allclose(merged, whole, atol=1e-13)
        np.testing.assert_allclose(m + np.log(w1 + w2), lse, atol=1e-13)


@pytest.mark.parametrize("heads", [(1, 1), (4, 2)])
def test_library_sdpa_cross_check(oracle, heads):
    # torch's scaled_dot_product_attention in fp64 with an explicit boolean mask
    Hq, Hkv = heads
    rng = np.random.default_rng(9)
    L, k, D = 15, 3, 16
    q, kc, v, qi, ki = _random_case(rng, [L], [k], Hq, Hkv, D, F32)
    scale = 1.0 / np.sqrt(D)
    out = oracle.verify_attention(q, kc, v, qi, ki, Hq, Hkv, D, scale, F32)
    G = Hq // Hkv
    tq = torch.from_numpy(q.astype(np.float64)).permute(1, 0, 2)[None]              # [1,Hq,R,D]
    tk = torch.from_numpy(kc.astype(np.float64)).repeat_interleave(G, 1).permute(1, 0, 2)[None]
    tv = torch.from_numpy(v.astype(np.float64)).repeat_interleave(G, 1).permute(1, 0, 2)[None]
    R = k + 1
    mask = torch.arange(L)[None, :] <= (L - R + torch.arange(R))[:, None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale)
    np.testing.assert_allclose(out, ref[0].permute(1, 0, 2).numpy(), atol=1e-12)


def test_rejects_bad_shapes(oracle):
    rng = np.random.default_rng(10)
    q, kc, v, qi, ki = _random_case(rng, [4], [3], 2, 1, 4, F32)
    oracle.verify_attention(q, kc, v, qi, ki, 2, 1, 4, 1.0, F32)
    with pytest.raises(RuntimeError):       # cache shorter than the k+1 new tokens
        oracle.verify_attention(q, kc[:3], v[:3], qi, np.array([0, 3]), 2, 1, 4, 1.0, F32)
    lib = oracle._load()
    assert lib.respec_oracle_verify_attention(None, None, None, None, None, None, None,
                                              1, 2, 1, 4, 1.0, 0, 1) != 0      # null pointers
    qp, kp, vp = (a.ctypes.data for a in (q, kc, v))
    qip = np.ascontiguousarray(qi, dtype=np.int32)
    kip = np.ascontiguousarray(ki, dtype=np.int64)
    out = np.zeros(q.shape)
    assert lib.respec_oracle_verify_attention(qp, kp, vp, qip.ctypes.data, kip.ctypes.data,
                                              out.ctypes.data, None, 1, 3, 2, 4, 1.0, 0, 1) != 0
