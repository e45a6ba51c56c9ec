"""GPU parity of respec_kd_rows (reward-weighted KD per logits row, Section 5.3) against the
CPU oracle.

Tolerances (derived from the arithmetic: p and q are formed in the log2 domain in fp32, where
an exponent of magnitude up to ~40 carries an absolute rounding error of ~2e-6, so p and q have
a relative error of a few 1e-6; the KL terms are summed in fp32 over at most 40 terms per thread
and in fp64 from there on):
  row loss   |gpu - ref| <= 2e-5 * (|ref| + 0.05 * w)
  gradient   f32:  |gpu - ref| <= 5e-6 * w
             bf16: |gpu - ref| <= 2^-8 * |ref| + 5e-6 * w     (the output is rounded to bf16)
  total      relative 2e-5.
"""
import numpy as np
import pytest
import torch

from helpers import env_setting
from paper_2510_26475_amd import binding, synth

pytestmark = pytest.mark.gpu


def _inputs(rows, V, dtype, seed, sigma=1.0, zero_rows=(), pad=0):
    g = torch.Generator(device="cuda").manual_seed(seed)
    dt = torch.float32 if dtype == "f32" else torch.bfloat16
    ld = V + pad
    t32 = 3.0 * torch.randn((rows, ld), generator=g, device="cuda")
    d32 = t32 + sigma * torch.randn((rows, ld), generator=g, device="cuda")
    target, draft = t32.to(dt)[:, :V], d32.to(dt)[:, :V]
    w = 0.1 + 1.9 * torch.rand((rows,), generator=g, device="cuda")
    for r in zero_rows:
        w[r] = 0.0
    return target, draft, w


def gpu_kd(target, draft, w, pad=0):
    rows, V = target.shape
    dt = binding.RESPEC_F32 if target.dtype == torch.float32 else binding.RESPEC_BF16
    ws = torch.empty(binding.respec_kd_rows_workspace_bytes(rows, V, dt), dtype=torch.uint8, device="cuda")
    grad = torch.full((rows, V + pad), float("nan"), dtype=target.dtype, device="cuda")[:, :V]
    loss = torch.full((rows,), float("nan"), dtype=torch.float32, device="cuda")
    total = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda")
    binding.respec_kd_rows(target, draft, w, grad, loss, total, ws)
    torch.cuda.synchronize()
    return grad, loss, total


def _parity(oracle, target, draft, w, pad=0):
    grad, loss, total = gpu_kd(target, draft, w, pad)
    odt = oracle.F32 if target.dtype == torch.float32 else oracle.BF16
    r_grad, r_loss, r_total = oracle.kd_rows(synth.to_host_array(target.contiguous()),
                                             synth.to_host_array(draft.contiguous()), w.cpu().numpy(), odt, n_threads=0)
    wh = w.double().cpu().numpy()
    g = grad.double().cpu().numpy()
    assert np.isfinite(g).all() and np.isfinite(loss.cpu().numpy()).all()
    gtol = 5e-6 * wh[:, None] + (2.0 ** -8 * np.abs(r_grad) if target.dtype == torch.bfloat16 else 0.0)
    gerr = np.abs(g - r_grad)
    assert (gerr <= gtol).all(), f"gradient error {gerr.max():.3e} (worst excess {(gerr - gtol).max():.3e})"
    lerr = np.abs(loss.double().cpu().numpy() - r_loss)
    assert (lerr <= 2e-5 * (np.abs(r_loss) + 0.05 * wh)).all(), f"row loss error {lerr.max():.3e}"
    assert abs(float(total) - r_total) <= 2e-5 * abs(r_total) + 1e-9
    return grad, loss, total, r_loss


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V", [8, 1024, 4096, 20480, 40960])
def test_small_and_medium_vocabularies(oracle, dtype, V):
    # from a row smaller than one batch of slots to rows of several batches with a ragged tail
    target, draft, w = _inputs(37, V, dtype, seed=V)
    _parity(oracle, target, draft, w)


@pytest.mark.parametrize("sigma", [0.5, 2.0])
def test_full_vocab_bf16(oracle, sigma):
    target, draft, w = _inputs(300, 151936, "bf16", seed=int(10 * sigma), sigma=sigma)
    _, _, _, r_loss = _parity(oracle, target, draft, w)
    assert (r_loss > 0).all()


def test_full_vocab_f32(oracle):
    target, draft, w = _inputs(40, 151936, "f32", seed=3)
    _parity(oracle, target, draft, w)


def test_rows_with_weight_zero_are_not_read_and_get_a_zero_gradient(oracle):
    target, draft, w = _inputs(50, 151936, "bf16", seed=4, zero_rows=(0, 7, 8, 9, 49))
    target[7] = float("nan")               # would poison the row's loss if it were read
    draft[49] = float("nan")
    grad, loss, total = gpu_kd(target, draft, w)
    for r in (0, 7, 8, 9, 49):
        assert float(loss[r]) == 0.0 and not grad[r].any()
    assert np.isfinite(float(total))
    keep = [r for r in range(50) if r not in (0, 7, 8, 9, 49)]
    idx = torch.tensor(keep, device="cuda")
    _, r_loss, r_total = oracle.kd_rows(synth.to_host_array(target[idx].contiguous()),
                                        synth.to_host_array(draft[idx].contiguous()), w[idx].cpu().numpy(),
                                        oracle.BF16, n_threads=0)
    assert abs(float(total) - r_total) <= 2e-5 * r_total


def test_row_strides_larger_than_the_vocabulary(oracle):
    target, draft, w = _inputs(20, 4096, "bf16", seed=5, pad=64)
    assert target.stride(0) == 4096 + 64
    _parity(oracle, target, draft, w, pad=8)


@pytest.mark.parametrize("wgs", [1, 3, 700])
def test_any_number_of_work_groups(oracle, wgs):
    target, draft, w = _inputs(70, 151936, "bf16", seed=6 + wgs % 97)
    with env_setting("RESPEC_KD_WGS", wgs):
        _parity(oracle, target, draft, w)


def test_a_vocabulary_wider_than_any_model_on_the_list(oracle):
    target, draft, w = _inputs(3, 400000, "bf16", seed=12)
    _parity(oracle, target, draft, w)


def test_identical_drafter_and_masked_tokens(oracle):
    target, _, w = _inputs(16, 151936, "bf16", seed=7)
    grad, loss, total = gpu_kd(target, target.clone(), w)
    assert float(loss.abs().max()) <= 2e-5 * 0.05 * 2.0 and float(grad.float().abs().max()) <= 1e-5
    target[:, 1000:2000] = float("-inf")    # tokens the target never emits
    _, draft, _ = _inputs(16, 151936, "bf16", seed=8)
    _parity(oracle, target, draft, w)


def test_runs_are_bitwise_reproducible():
    target, draft, w = _inputs(64, 151936, "bf16", seed=9)
    a, b = gpu_kd(target, draft, w), gpu_kd(target, draft, w)
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.int16) if x.dtype == torch.bfloat16 else x, y.view(torch.int16) if y.dtype == torch.bfloat16 else y)


def test_bad_arguments_are_rejected_before_any_launch():
    target, draft, w = _inputs(4, 1024, "f32", seed=1)
    grad = torch.empty_like(target)
    loss = torch.empty(4, device="cuda")
    ws = torch.empty(binding.respec_kd_rows_workspace_bytes(4, 1024, binding.RESPEC_F32), dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.RespecError) as e:
        binding.respec_kd_rows(target, draft, w, grad, loss, None, ws[:128])
    assert e.value.status == 3
    t2, d2, _ = _inputs(4, 1022, "f32", seed=1)          # rows are not whole 16-byte pieces
    with pytest.raises(binding.RespecError) as e:
        binding.respec_kd_rows(t2.contiguous(), d2.contiguous(), w, torch.empty((4, 1022), device="cuda"), loss, None, ws)
    assert e.value.status == 2
