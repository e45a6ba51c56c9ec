"""Pins for the oracle's greedy verification and per-sequence temperature (CPU only).

Temperature 0 is the T -> 0 limit of Section 2.2's validation: softmax(z/T) tends to a point
mass on the largest logit, so Eq. 1 accepts a drafted token iff it is the target's argmax and
Eq. 2 replaces it by that argmax.  Pinned against numpy's argmax (a library routine that returns
the first maximum), against the stochastic oracle at a tiny temperature on well separated
logits, and, for batches that mix temperatures, against the one-temperature function.
"""
import numpy as np
import pytest
import torch

F32, BF16 = 0, 1


def _indptr(ks):
    out = [0]
    for k in ks:
        out.append(out[-1] + k + 1)
    return np.array(out, dtype=np.int32)


def _bf16_bits(x32):
    t = torch.from_numpy(np.ascontiguousarray(x32, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def _bf16_to_f32(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32)


def _reference_greedy(target, tokens, ks, max_k):
    """Written from the definition with numpy's argmax; `target` holds real numbers."""
    B = len(ks)
    out = np.full((B, max_k + 1), -1, dtype=np.int32)
    n_acc = np.zeros(B, dtype=np.int32)
    row = drow = 0
    for b, k in enumerate(ks):
        n = 0
        while n < k and tokens[drow + n] == int(np.argmax(target[row + n])):
            out[b, n] = tokens[drow + n]
            n += 1
        out[b, n] = int(np.argmax(target[row + n]))
        n_acc[b] = n
        row += k + 1
        drow += k
    return out, n_acc


@pytest.mark.parametrize("dtype", [F32, BF16])
def test_equals_numpy_argmax_row_by_row(oracle, dtype):
    rng = np.random.default_rng(5 + dtype)
    ks = [0, 3, 1, 5, 2, 4, 0, 5]
    V, max_k = 97, 5
    total_q = sum(ks) + len(ks)
    t32 = rng.normal(0, 3, (total_q, V)).astype(np.float32)
    target = t32 if dtype == F32 else _bf16_bits(t32)
    real = t32 if dtype == F32 else _bf16_to_f32(target)
    # drafted tokens: the argmax (accepted) most of the time, something else now and then
    tokens, row = [], 0
    for k in ks:
        for i in range(k):
            a = int(np.argmax(real[row + i]))
            tokens.append(a if rng.random() < 0.7 else int(rng.integers(0, V)))
        row += k + 1
    tokens = np.array(tokens, dtype=np.int32)
    temps = np.zeros(len(ks), dtype=np.float32)
    u_final = np.full(len(ks), np.nan, dtype=np.float32)       # never read
    toks, n, flags = oracle.rejection_sample_per_seq(target, None, tokens, _indptr(ks), None, u_final, max_k,
                                                     temps, dtype)
    r_toks, r_n = _reference_greedy(real, tokens, ks, max_k)
    assert np.array_equal(n, r_n) and np.array_equal(toks, r_toks)
    assert not flags.any()
    assert 0 < n.sum() < sum(ks)          # both outcomes occur


def test_ties_go_to_the_lowest_token_id(oracle):
    V = 16
    target = np.zeros((3, V), dtype=np.float32)
    target[0, [4, 9]] = 2.0        # tie between 4 and 9
    target[1, [9, 4]] = 2.0
    target[2, 7] = 1.0
    # sequence 0 drafts 4 (the first maximum: accepted) then 9 (tied, but not the first: rejected)
    toks, n, _ = oracle.rejection_sample_per_seq(target, None, np.array([4, 9], dtype=np.int32), _indptr([2]), None,
                                                 np.zeros(1, np.float32), 2, np.zeros(1, np.float32), F32)
    assert n.tolist() == [1] and toks.tolist() == [[4, 4, -1]]
    # bf16 rounding creates ties that fp32 would not have
    z = np.zeros((1, V), dtype=np.float32)
    z[0, 3], z[0, 11] = 8.0, 8.01          # both round to 8.0 in bf16
    toks, n, _ = oracle.rejection_sample_per_seq(_bf16_bits(z), None, None, _indptr([0]), None,
                                                 np.zeros(1, np.float32), 0, np.zeros(1, np.float32), BF16)
    assert toks.tolist() == [[3]] and n.tolist() == [0]


def test_is_the_small_temperature_limit_of_eq1_and_eq2(oracle):
    """Logits whose largest entry leads by at least 1: at T = 0.01 the softmax puts all but
    e^-100 of its mass on the argmax, so the stochastic procedure (any uniforms below 0.99)
    must take the greedy decisions."""
    rng = np.random.default_rng(11)
    ks = [4, 4, 2, 0, 3, 4, 1, 4]
    V, max_k = 64, 4
    total_q, n_draft = sum(ks) + len(ks), sum(ks)
    target = np.stack([rng.permutation(V) for _ in range(total_q)]).astype(np.float32)
    draft = np.stack([rng.permutation(V) for _ in range(n_draft)]).astype(np.float32)
    # the drafter proposes its own argmax; make it agree with the target on most rows
    row, drow = 0, 0
    for k in ks:
        for i in range(k):
            if rng.random() < 0.75:
                draft[drow + i] = target[row + i]
        row += k + 1
        drow += k
    tokens = np.argmax(draft, axis=1).astype(np.int32)
    u_acc = rng.uniform(0, 0.99, n_draft).astype(np.float32)
    u_fin = rng.uniform(0, 0.99, len(ks)).astype(np.float32)
    s_toks, s_n, _ = oracle.rejection_sample(target, draft, tokens, _indptr(ks), u_acc, u_fin, max_k, 0.01, F32)
    g_toks, g_n, g_f = oracle.rejection_sample_per_seq(target, draft, tokens, _indptr(ks), u_acc, u_fin, max_k,
                                                       np.zeros(len(ks), np.float32), F32)
    assert np.array_equal(s_n, g_n) and np.array_equal(s_toks, g_toks)
    assert 0 < g_n.sum() < n_draft and not g_f.any()


def test_mixed_temperatures_equal_the_one_temperature_function_per_sequence(oracle):
    rng = np.random.default_rng(3)
    ks = [3, 0, 2, 3, 1, 3]
    temps = np.array([0.6, 0.0, 1.0, 0.0, 0.4, 0.6], dtype=np.float32)
    V, max_k = 50, 3
    total_q, n_draft = sum(ks) + len(ks), sum(ks)
    target = rng.normal(0, 3, (total_q, V)).astype(np.float32)
    draft = (target[[r for b, k in enumerate(ks) for r in range(_indptr(ks)[b], _indptr(ks)[b] + k)]]
             + rng.normal(0, 1, (n_draft, V))).astype(np.float32)
    tokens = rng.integers(0, V, n_draft).astype(np.int32)
    # greedy sequences draft the target's argmax half of the time
    ip = _indptr(ks)
    for b, k in enumerate(ks):
        if temps[b] == 0:
            for i in range(k):
                if rng.random() < 0.5:
                    tokens[ip[b] - b + i] = int(np.argmax(target[ip[b] + i]))
    u_acc = rng.uniform(0, 1, n_draft).astype(np.float32)
    u_fin = rng.uniform(0, 1, len(ks)).astype(np.float32)
    toks, n, flags = oracle.rejection_sample_per_seq(target, draft, tokens, ip, u_acc, u_fin, max_k, temps, F32)
    for b, k in enumerate(ks):
        r0, d0 = ip[b], ip[b] - b
        t_b, d_b, x_b = target[r0:r0 + k + 1], draft[d0:d0 + k], tokens[d0:d0 + k]
        if temps[b] > 0:
            e_toks, e_n, e_f = oracle.rejection_sample(t_b, d_b if k else None, x_b if k else None, _indptr([k]),
                                                       u_acc[d0:d0 + k] if k else None, u_fin[b:b + 1], max_k,
                                                       float(temps[b]), F32)
        else:
            e_toks, e_n = _reference_greedy(t_b, x_b, [k], max_k)
            e_f = np.zeros(1, np.int32)
        assert n[b] == e_n[0] and toks[b].tolist() == e_toks[0].tolist() and flags[b] == e_f[0], b


def test_greedy_reads_nothing_after_the_first_rejection_and_no_drafter_data(oracle):
    rng = np.random.default_rng(8)
    V, k = 40, 4
    target = rng.normal(0, 3, (k + 1, V)).astype(np.float32)
    tokens = np.argmax(target[:k], axis=1).astype(np.int32)
    tokens[1] = (tokens[1] + 1) % V                      # rejected at position 1
    target[2:] = np.nan                                  # rows after the rejection
    draft = np.full((k, V), np.nan, dtype=np.float32)
    nan_u = np.full(k, np.nan, dtype=np.float32)
    toks, n, _ = oracle.rejection_sample_per_seq(target, draft, tokens, _indptr([k]), nan_u,
                                                 np.full(1, np.nan, np.float32), k, np.zeros(1, np.float32), F32)
    assert n.tolist() == [1]
    assert toks.tolist() == [[int(tokens[0]), int(np.argmax(target[1])), -1, -1, -1]]


def test_all_accepted_emits_the_argmax_of_the_bonus_row_and_k0_is_plain_greedy_decoding(oracle):
    rng = np.random.default_rng(9)
    V, k = 33, 3
    target = rng.normal(0, 3, (k + 1, V)).astype(np.float32)
    tokens = np.argmax(target[:k], axis=1).astype(np.int32)
    toks, n, _ = oracle.rejection_sample_per_seq(target, None, tokens, _indptr([k]), None, np.zeros(1, np.float32), k,
                                                 np.zeros(1, np.float32), F32)
    assert n.tolist() == [k] and toks.tolist() == [tokens.tolist() + [int(np.argmax(target[k]))]]
    toks, n, _ = oracle.rejection_sample_per_seq(target[:1], None, None, _indptr([0]), None, np.zeros(1, np.float32), 0,
                                                 np.zeros(1, np.float32), F32)
    assert n.tolist() == [0] and toks.tolist() == [[int(np.argmax(target[0]))]]


def test_bad_temperatures_are_errors(oracle):
    target = np.zeros((1, 8), dtype=np.float32)
    for bad in (-1.0, np.nan, np.inf):
        with pytest.raises(RuntimeError):
            oracle.rejection_sample_per_seq(target, None, None, _indptr([0]), None, np.zeros(1, np.float32), 0,
                                            np.array([bad], np.float32), F32)
