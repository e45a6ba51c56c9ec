"""Pins for the rejection-sampling oracle (CPU only).

The oracle walks Section 2.2's validation step by step (Eq. 1 acceptance, Eq. 2 residual).
Here it is pinned against what the paper and the mathematics fix: a hand-worked case,
q == p, k = 0 against numpy's cumsum/searchsorted sampler, the losslessness claim (the
emitted-token marginal is p) by chi-square and by exact enumeration, the closed-form
acceptance rate 1 - TV(p,q), disjoint supports and extreme uniforms.
"""
import json
import os

import numpy as np
import pytest
import torch
from scipy import special, stats

F32, BF16 = 0, 1
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _indptr(ks):
    out = [0]
    for k in ks:
        out.append(out[-1] + k + 1)
    return np.array(out, dtype=np.int32)


def _bf16_bits(x32):
    t = torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def _bf16_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _softmax64(z, T=1.0):
    return special.softmax(np.asarray(z, dtype=np.float64) / float(np.float32(T)), axis=-1)


def _numpy_inverse_cdf(p, u):
    """Library sampler: first index whose cumulative sum exceeds u (side='right')."""
    return int(np.searchsorted(np.cumsum(p, dtype=np.float64), u, side="right"))


def _tile_rows(row, n):
    return np.ascontiguousarray(np.broadcast_to(row, (n, row.shape[-1])), dtype=np.float32)


# --------------------------------------------------------------------------------------
def test_hand_worked_case_from_eq1_eq2(oracle):
    g = json.load(open(os.path.join(GOLDEN, "eq1_eq2_hand_case.json")))
    tl = np.log(np.array(g["target_logits_are_log_of"], dtype=np.float64)).astype(np.float32)
    dl = np.log(np.array(g["draft_logits_are_log_of"], dtype=np.float64)).astype(np.float32)
    p = oracle.softmax_rows(tl[None], 1.0, F32)[0]
    np.testing.assert_allclose(p, g["p"], atol=1e-7)
    np.testing.assert_allclose(oracle.softmax_rows(dl[None], 1.0, F32)[0], g["q"], atol=1e-7)
    for case in g["cases"]:
        toks, n, flags = oracle.rejection_sample(
            _tile_rows(tl, 2), dl[None], np.array([case["draft_token"]]), _indptr([1]),
            np.array([case["u_accept"]], dtype=np.float32),
            np.array([case["u_final"]], dtype=np.float32), 1, 1.0, F32)
        if case["u_final"] == 0.5:       # sits on a CDF edge: flagged, either neighbour is valid
            assert flags[0] & 2 and toks[0, 1] in (1, 2) and n[0] == 1
            continue
        assert n[0] == case["num_accepted"], case["why"]
        assert toks[0].tolist() == case["tokens"], case["why"]


def test_softmax_matches_scipy_with_temperature_and_bf16(oracle):
    rng = np.random.default_rng(0)
    z = (3.0 * rng.standard_normal((5, 333))).astype(np.float32)
    for T in (1.0, 0.6, 0.4):
        np.testing.assert_allclose(oracle.softmax_rows(z, T, F32), _softmax64(z, T), rtol=1e-12)
    zb = _bf16_bits(z)
    np.testing.assert_allclose(oracle.softmax_rows(zb, 0.6, BF16),
                               _softmax64(_bf16_to_f64(zb), 0.6), rtol=1e-12)


def test_identical_drafter_accepts_every_draft(oracle):
    rng = np.random.default_rng(1)
    V, ks = 257, [4, 1, 3, 0, 4]
    qi = _indptr(ks)
    B, total = len(ks), int(qi[-1])
    target = (3.0 * rng.standard_normal((total, V))).astype(np.float32)
    drows = np.concatenate([np.arange(qi[b], qi[b] + ks[b]) for b in range(B)]).astype(int)
    draft = target[drows].copy()
    toks_in = rng.integers(0, V, size=len(drows)).astype(np.int32)
    u_acc = np.full(len(drows), np.float32(1.0) - np.float32(2.0 ** -24))   # largest u below 1
    u_fin = rng.random(B).astype(np.float32)
    toks, n, flags = oracle.rejection_sample(target, draft, toks_in, qi, u_acc, u_fin, 4, 0.6, F32)
    assert n.tolist() == ks
    p = _softmax64(target, 0.6)
    for b in range(B):
        d0 = qi[b] - b
        assert toks[b, :ks[b]].tolist() == toks_in[d0:d0 + ks[b]].tolist()
        if not flags[b] & 2:
            assert toks[b, ks[b]] == _numpy_inverse_cdf(p[qi[b] + ks[b]], u_fin[b])
        assert (toks[b, ks[b] + 1:] == -1).all()


@pytest.mark.parametrize("dtype,T", [(F32, 1.0), (F32, 0.6), (BF16, 1.0)])
def test_no_draft_is_ordinary_sampling(oracle, dtype, T):
    rng = np.random.default_rng(2)
    B, V = 400, 1024
    z = (3.0 * rng.standard_normal((B, V))).astype(np.float32)
    stored = z if dtype == F32 else _bf16_bits(z)
    u = rng.random(B).astype(np.float32)
    toks, n, flags = oracle.rejection_sample(stored, None, None, _indptr([0] * B), None, u, 0, T,
                                             dtype)
    p = _softmax64(z if dtype == F32 else _bf16_to_f64(stored), T)
    assert (n == 0).all() and toks.shape == (B, 1)
    unflagged = [b for b in range(B) if not flags[b] & 2]
    assert len(unflagged) > 0.9 * B
    for b in unflagged:
        assert toks[b, 0] == _numpy_inverse_cdf(p[b], float(u[b]))


def _draw_from(rng, probs, n):
    return rng.choice(len(probs), size=n, p=probs).astype(np.int32)


def test_chi_square_emitted_marginal_is_target(oracle):
    """Losslessness (Section 2.2, after Eq. 2): 10^6 draws, k = 1, tiny vocabulary."""
    rng = np.random.default_rng(3)
    V, N = 12, 1_000_000
    t_row = (1.5 * rng.standard_normal(V)).astype(np.float32)
    d_row = (t_row + rng.standard_normal(V)).astype(np.float32)
    p, q = _softmax64(t_row), _softmax64(d_row)
    qi = _indptr([1] * N)
    toks, n, _ = oracle.rejection_sample(
        _tile_rows(t_row, 2 * N), _tile_rows(d_row, N), _draw_from(rng, q, N), qi,
        rng.random(N).astype(np.float32), rng.random(N).astype(np.float32), 1, 1.0, F32,
        n_threads=0)
    counts = np.bincount(toks[:, 0], minlength=V)
    chi2, pval = stats.chisquare(counts, p * N)
    assert pval > 1e-3, (chi2, pval)
    # acceptance rate has the closed form sum_x min(p,q) = 1 - TV(p,q)
    alpha = np.minimum(p, q).sum()
    assert abs(n.mean() - alpha) < 4.0 * np.sqrt(alpha * (1 - alpha) / N)
    # and the drafter's own marginal would fail the same test: the test has power
    assert stats.chisquare(np.bincount(_draw_from(rng, q, N), minlength=V), p * N)[1] < 1e-6


def test_chi_square_every_emitted_slot_k3(oracle):
    """With independent rows, slot j (given that it is emitted) is distributed as p_j."""
    rng = np.random.default_rng(4)
    V, N, k = 9, 400_000, 3
    t_rows = (1.5 * rng.standard_normal((k + 1, V))).astype(np.float32)
    d_rows = (t_rows[:k] + 0.8 * rng.standard_normal((k, V))).astype(np.float32)
    p, q = _softmax64(t_rows), _softmax64(d_rows)
    target = np.ascontiguousarray(np.broadcast_to(t_rows, (N, k + 1, V))).reshape(-1, V)
    draft = np.ascontiguousarray(np.broadcast_to(d_rows, (N, k, V))).reshape(-1, V)
    d_toks = np.stack([_draw_from(rng, q[i], N) for i in range(k)], axis=1).reshape(-1)
    toks, n, _ = oracle.rejection_sample(
        target, draft, d_toks, _indptr([k] * N), rng.random(N * k).astype(np.float32),
        rng.random(N).astype(np.float32), k, 1.0, F32, n_threads=0)
    alpha = np.minimum(p[:k], q).sum(axis=1)
    for j in range(k + 1):
        emitted = toks[:, j] >= 0
        assert (emitted == (n >= j)).all()
        want = N * np.prod(alpha[:j])
        assert abs(emitted.sum() - want) < 5.0 * np.sqrt(want)
        counts = np.bincount(toks[emitted, j], minlength=V)
        assert stats.chisquare(counts, p[j] * emitted.sum())[1] > 1e-3, j
    # expected emitted tokens per step: 1 + a0 + a0 a1 + a0 a1 a2
    want_len = 1 + alpha[0] + alpha[0] * alpha[1] + alpha[0] * alpha[1] * alpha[2]
    assert abs((n + 1).mean() - want_len) < 0.01


def test_exact_enumeration_on_a_uniform_grid(oracle):
    """sum_x q(x) [ a(x) delta_x + (1 - a(x)) r ] = p, with u replaced by a fine midpoint grid."""
    rng = np.random.default_rng(5)
    V, M = 4, 400
    t_row = rng.standard_normal(V).astype(np.float32)
    d_row = rng.standard_normal(V).astype(np.float32)
    p, q = _softmax64(t_row), _softmax64(d_row)
    grid = ((np.arange(M) + 0.5) / M).astype(np.float32)
    ua, uf = np.meshgrid(grid, grid, indexing="ij")
    N = M * M
    emitted = np.zeros(V)
    for x in range(V):
        toks, n, _ = oracle.rejection_sample(
            _tile_rows(t_row, 2 * N), _tile_rows(d_row, N), np.full(N, x, dtype=np.int32),
            _indptr([1] * N), ua.reshape(-1), uf.reshape(-1), 1, 1.0, F32, n_threads=0)
        emitted += q[x] * np.bincount(toks[:, 0], minlength=V) / N
        rho = min(1.0, p[x] / q[x])
        assert abs(n.mean() - rho) <= 1.0 / M + 1e-12           # Eq. 1 on the grid
    np.testing.assert_allclose(emitted, p, atol=2.0 / M)


def test_residual_when_supports_are_disjoint(oracle):
    rng = np.random.default_rng(6)
    V, B = 64, 200
    t = (2.0 * rng.standard_normal((2 * B, V))).astype(np.float32)
    d = (2.0 * rng.standard_normal((B, V))).astype(np.float32)
    t[:, 1::2] = -np.inf        # target lives on even ids
    d[:, 0::2] = -np.inf        # drafter lives on odd ids
    d_toks = (2 * rng.integers(0, V // 2, size=B) + 1).astype(np.int32)
    u_fin = rng.random(B).astype(np.float32)
    toks, n, flags = oracle.rejection_sample(t, d, d_toks, _indptr([1] * B),
                                             np.zeros(B, dtype=np.float32), u_fin, 1, 1.0, F32)
    assert (n == 0).all()                       # p(x) = 0 is rejected even at u = 0
    p = _softmax64(t[0::2])
    for b in range(B):
        if not flags[b] & 2:
            assert toks[b, 0] == _numpy_inverse_cdf(p[b], float(u_fin[b]))   # residual == p
        assert toks[b, 0] % 2 == 0 and toks[b, 1] == -1


def test_extreme_uniforms(oracle):
    rng = np.random.default_rng(7)
    V, B = 50, 300
    t = (2.0 * rng.standard_normal((2 * B, V))).astype(np.float32)
    d = (2.0 * rng.standard_normal((B, V))).astype(np.float32)
    d_toks = rng.integers(0, V, size=B).astype(np.int32)
    qi = _indptr([1] * B)
    u_fin = rng.random(B).astype(np.float32)
    _, n0, _ = oracle.rejection_sample(t, d, d_toks, qi, np.zeros(B, dtype=np.float32), u_fin, 1,
                                       1.0, F32)
    assert (n0 == 1).all()                      # u = 0 accepts whenever p(x) > 0
    big = np.full(B, np.float32(1.0) - np.float32(2.0 ** -24))
    _, n1, _ = oracle.rejection_sample(t, d, d_toks, qi, big, u_fin, 1, 1.0, F32)
    p, q = _softmax64(t[0::2]), _softmax64(d)
    rho = p[np.arange(B), d_toks] / q[np.arange(B), d_toks]
    clear = np.abs(np.minimum(rho, 1.0) - big) > 1e-6
    assert ((n1 == 1) == (rho >= 1.0))[clear].all()


def test_residual_token_has_positive_residual_mass_and_matches_numpy(oracle):
    rng = np.random.default_rng(8)
    V, B = 300, 500
    t = (3.0 * rng.standard_normal((2 * B, V))).astype(np.float32)
    d = (t[0::2] + rng.standard_normal((B, V))).astype(np.float32)
    q = _softmax64(d)
    p = _softmax64(t[0::2])
    d_toks = np.array([rng.choice(V, p=q[b]) for b in range(B)], dtype=np.int32)
    u_acc, u_fin = rng.random(B).astype(np.float32), rng.random(B).astype(np.float32)
    toks, n, flags = oracle.rejection_sample(t, d, d_toks, _indptr([1] * B), u_acc, u_fin, 1, 1.0,
                                             F32)
    rejected = np.flatnonzero(n == 0)
    assert 0.2 * B < len(rejected) < 0.6 * B
    for b in rejected:
        w = np.maximum(p[b] - q[b], 0.0)
        # residual identity: the two one-sided masses are both the total-variation distance
        assert abs(w.sum() - np.maximum(q[b] - p[b], 0.0).sum()) < 1e-12
        assert w.sum() >= q[b, d_toks[b]] - p[b, d_toks[b]] > 0
        assert w[toks[b, 0]] > 0
        if not flags[b] & 2:
            assert toks[b, 0] == _numpy_inverse_cdf(w / w.sum(), float(u_fin[b]))
    for b in np.flatnonzero(n == 1):
        if not flags[b] & 2:
            assert toks[b, 1] == _numpy_inverse_cdf(_softmax64(t[2 * b + 1]), float(u_fin[b]))


def test_rows_after_the_first_rejection_are_never_read(oracle):
    rng = np.random.default_rng(9)
    V, ks = 128, [4, 3, 4, 2, 0, 4]
    qi = _indptr(ks)
    B, total = len(ks), int(qi[-1])
    t = (3.0 * rng.standard_normal((total, V))).astype(np.float32)
    drow = np.concatenate([np.arange(qi[b], qi[b] + ks[b]) for b in range(B)]).astype(int)
    d = (t[drow] + 1.5 * rng.standard_normal((len(drow), V))).astype(np.float32)
    q = _softmax64(d)
    d_toks = np.array([rng.choice(V, p=q[r]) for r in range(len(drow))], dtype=np.int32)
    u_acc, u_fin = rng.random(len(drow)).astype(np.float32), rng.random(B).astype(np.float32)
    base = oracle.rejection_sample(t, d, d_toks, qi, u_acc, u_fin, 4, 1.0, F32)
    assert len(set(base[1].tolist())) > 2
    t2, d2, u2, tok2 = t.copy(), d.copy(), u_acc.copy(), d_toks.copy()
    for b in range(B):
        n = int(base[1][b])
        t2[qi[b] + n + 1: qi[b + 1]] = np.nan
        d0 = qi[b] - b
        d2[d0 + n + 1: d0 + ks[b]] = np.nan
        u2[d0 + n + 1: d0 + ks[b]] = np.nan
        tok2[d0 + n + 1: d0 + ks[b]] = 0
    again = oracle.rejection_sample(t2, d2, tok2, qi, u2, u_fin, 4, 1.0, F32)
    for a, b_ in zip(base, again):
        np.testing.assert_array_equal(a, b_)


def test_batched_ragged_call_equals_one_sequence_at_a_time(oracle):
    rng = np.random.default_rng(10)
    V, ks = 97, [3, 0, 5, 1, 2]
    qi = _indptr(ks)
    B, total = len(ks), int(qi[-1])
    t = (3.0 * rng.standard_normal((total, V))).astype(np.float32)
    d = (3.0 * rng.standard_normal((total - B, V))).astype(np.float32)
    d_toks = rng.integers(0, V, size=total - B).astype(np.int32)
    u_acc = (0.3 * rng.random(total - B)).astype(np.float32)
    u_fin = rng.random(B).astype(np.float32)
    toks, n, flags = oracle.rejection_sample(t, d, d_toks, qi, u_acc, u_fin, 5, 0.6, F32)
    for b in range(B):
        k, d0 = ks[b], qi[b] - b
        tb, nb, fb = oracle.rejection_sample(
            t[qi[b]:qi[b + 1]], d[d0:d0 + k] if k else None, d_toks[d0:d0 + k] if k else None,
            _indptr([k]), u_acc[d0:d0 + k] if k else None, u_fin[b:b + 1], k, 0.6, F32)
        assert nb[0] == n[b] and fb[0] == flags[b]
        assert tb[0].tolist() == toks[b, :k + 1].tolist()
        assert (toks[b, k + 1:] == -1).all()


def test_boundary_flags(oracle):
    # u exactly on the acceptance ratio: not accepted (strict <) and flagged
    t = np.log(np.array([[1, 1, 2], [1, 1, 2]], dtype=np.float64)).astype(np.float32)
    d = np.log(np.array([[2, 1, 1]], dtype=np.float64)).astype(np.float32)
    toks, n, flags = oracle.rejection_sample(t, d, np.array([0]), _indptr([1]),
                                             np.array([0.5], dtype=np.float32),
                                             np.array([0.3], dtype=np.float32), 1, 1.0, F32)
    assert flags[0] & 1
    toks, n, flags = oracle.rejection_sample(t, d, np.array([0]), _indptr([1]),
                                             np.array([0.25], dtype=np.float32),
                                             np.array([0.3], dtype=np.float32), 1, 1.0, F32)
    assert n[0] == 1 and not flags[0] & 1 and toks[0, 0] == 0
    toks, n, flags = oracle.rejection_sample(t, d, np.array([0]), _indptr([1]),
                                             np.array([0.75], dtype=np.float32),
                                             np.array([0.3], dtype=np.float32), 1, 1.0, F32)
    # rejected: residual = max(0, p - q) = (0, 0, 1/4) / (1/4): token 2 whatever u is
    assert n[0] == 0 and toks[0].tolist() == [2, -1] and not flags[0] & 1


def test_rejects_bad_arguments(oracle):
    t = np.zeros((2, 8), dtype=np.float32)
    d = np.zeros((1, 8), dtype=np.float32)
    u = np.array([0.5], dtype=np.float32)
    with pytest.raises(RuntimeError):
        oracle.rejection_sample(t, d, np.array([8]), _indptr([1]), u, u, 1, 1.0, F32)   # token id
    with pytest.raises(RuntimeError):
        oracle.rejection_sample(t, d, np.array([0]), _indptr([1]), u, u, 1, 0.0, F32)   # T <= 0
    with pytest.raises(RuntimeError):
        oracle.rejection_sample(t, d, np.array([0]), _indptr([1]), u, u, 0, 1.0, F32)   # k > max_k


def test_zero_uniform_skips_tokens_without_mass(oracle):
    # strict '>' in the inverse-CDF walk: u = 0 returns the first token with positive mass
    t = np.array([[-np.inf, -np.inf, 0.0, 1.0]], dtype=np.float32)
    toks, n, _ = oracle.rejection_sample(t, None, None, _indptr([0]), None,
                                         np.zeros(1, dtype=np.float32), 0, 1.0, F32)
    assert toks[0, 0] == 2 and n[0] == 0
