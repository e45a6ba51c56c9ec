"""Pins of the oracle's reward-weighted KD row function (CPU only; Section 5.3)."""
import numpy as np
import pytest
import torch
from scipy import special

from paper_2510_26475_amd import synth


def _rows(rows, V, seed, sigma=1.0, dtype=np.float32):
    g = np.random.default_rng(seed)
    t = (3.0 * g.standard_normal((rows, V))).astype(np.float32)
    d = (t + sigma * g.standard_normal((rows, V))).astype(np.float32)
    w = g.uniform(0.1, 2.0, rows).astype(np.float32)
    return t, d, w


def test_against_scipy_relative_entropy(oracle):
    t, d, w = _rows(7, 300, 1)
    grad, loss, total = oracle.kd_rows(t, d, w, oracle.F32)
    p = special.softmax(t.astype(np.float64), axis=1)
    q = special.softmax(d.astype(np.float64), axis=1)
    np.testing.assert_allclose(loss, w * special.rel_entr(p, q).sum(axis=1), rtol=1e-12)
    np.testing.assert_allclose(grad, w[:, None] * (q - p), rtol=0, atol=1e-15)
    assert abs(total - loss.sum()) <= 1e-12 * abs(total)


def test_against_torch_autograd_of_kl_div(oracle):
    t, d, w = _rows(5, 257, 2, sigma=2.0)
    zq = torch.tensor(d, dtype=torch.float64, requires_grad=True)
    logp = torch.log_softmax(torch.tensor(t, dtype=torch.float64), dim=1)
    kl = torch.nn.functional.kl_div(torch.log_softmax(zq, dim=1), logp, reduction="none", log_target=True).sum(dim=1)
    total_t = (torch.tensor(w, dtype=torch.float64) * kl).sum()
    total_t.backward()
    grad, loss, total = oracle.kd_rows(t, d, w, oracle.F32)
    np.testing.assert_allclose(total, float(total_t.detach()), rtol=1e-12)
    np.testing.assert_allclose(grad, zq.grad.numpy(), rtol=0, atol=1e-14)


def test_gradient_is_the_derivative_of_the_loss(oracle):
    """Central differences of a loss written here (log-sum-exp form), not of the oracle's."""
    t, d, w = _rows(2, 9, 3)

    def loss_of(zq):
        zp = t.astype(np.float64)
        lp = zp - special.logsumexp(zp, axis=1, keepdims=True)
        lq = zq - special.logsumexp(zq, axis=1, keepdims=True)
        return float((w * (np.exp(lp) * (lp - lq)).sum(axis=1)).sum())

    grad, _, _ = oracle.kd_rows(t, d, w, oracle.F32)
    z0 = d.astype(np.float64)
    eps = 1e-5
    for r in range(2):
        for x in range(9):
            zp_, zm_ = z0.copy(), z0.copy()
            zp_[r, x] += eps
            zm_[r, x] -= eps
            assert abs((loss_of(zp_) - loss_of(zm_)) / (2 * eps) - grad[r, x]) < 1e-8


def test_identical_drafter_has_no_loss_and_no_gradient(oracle):
    t, _, w = _rows(4, 100, 4)
    grad, loss, total = oracle.kd_rows(t, t.copy(), w, oracle.F32)
    assert np.abs(loss).max() < 1e-15 and np.abs(grad).max() < 1e-16 and abs(total) < 1e-14


def test_two_token_closed_form_and_weight_linearity(oracle):
    # p = (0.8, 0.2), q = (0.5, 0.5): KL = 0.8 ln 1.6 + 0.2 ln 0.4
    t = np.log(np.array([[0.8, 0.2]], dtype=np.float64)).astype(np.float32)
    d = np.zeros((1, 2), dtype=np.float32)
    p = special.softmax(t.astype(np.float64), axis=1)[0]      # what the float32 logits really encode
    kl = p[0] * np.log(p[0] / 0.5) + p[1] * np.log(p[1] / 0.5)
    for w in (1.0, 0.25, 3.0):
        grad, loss, _ = oracle.kd_rows(t, d, np.array([w], dtype=np.float32), oracle.F32)
        np.testing.assert_allclose(loss[0], w * kl, rtol=1e-13)
        np.testing.assert_allclose(grad[0], w * (0.5 - p), rtol=0, atol=1e-15)
    assert abs(kl - (0.8 * np.log(1.6) + 0.2 * np.log(0.4))) < 1e-7


def test_invariants_row_sums_shift_and_masked_tokens(oracle):
    t, d, w = _rows(6, 64, 5)
    t[:, 7] = -np.inf                      # a token the target never emits: no loss term, gradient = w q
    grad, loss, _ = oracle.kd_rows(t, d, w, oracle.F32)
    assert np.abs(grad.sum(axis=1)).max() < 1e-14
    q = special.softmax(d.astype(np.float64), axis=1)
    np.testing.assert_allclose(grad[:, 7], w * q[:, 7], rtol=1e-12)
    assert np.isfinite(loss).all() and (loss >= 0).all()
    # adding a constant to a row of either input changes nothing (up to the rounding of the shifted float32 inputs)
    g2, l2, _ = oracle.kd_rows(t + np.float32(1.0), d - np.float32(2.0), w, oracle.F32)
    np.testing.assert_allclose(l2, loss, rtol=1e-5)
    np.testing.assert_allclose(g2, grad, rtol=0, atol=1e-6)


def test_bf16_inputs_are_read_as_bf16(oracle):
    t, d, w = _rows(3, 128, 6)
    tb = torch.tensor(t).to(torch.bfloat16)
    db = torch.tensor(d).to(torch.bfloat16)
    g16, l16, _ = oracle.kd_rows(synth.to_host_array(tb), synth.to_host_array(db), w, oracle.BF16)
    g32, l32, _ = oracle.kd_rows(tb.float().numpy(), db.float().numpy(), w, oracle.F32)
    np.testing.assert_array_equal(g16, g32)
    np.testing.assert_array_equal(l16, l32)
