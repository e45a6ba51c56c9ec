"""The entry point that allocates nothing: respec_verify_attention_static, whose scratch is a
buffer inside the library's device image instead of a workspace argument.

It must give what respec_verify_attention gives (same kernels, same split: bit for bit), also on
a second call with a smaller batch right behind a larger one (the buffer keeps the first call's
contents), and it must refuse a batch whose scratch does not fit.  Called through the C ABI.
"""
import ctypes
import math

import pytest
import torch

from helpers import gpu_attention, oracle_attention
from paper_2510_26475_amd import binding, synth

pytestmark = pytest.mark.gpu


def _static_attention(batch):
    wl = batch.wl
    out = torch.full_like(batch.q, float("nan"))
    lse = torch.full((batch.total_q, wl.Hq), float("nan"), dtype=torch.float32, device=batch.q.device)
    binding.respec_verify_attention_static(batch.q, batch.k_cache, batch.v_cache, batch.q_indptr, batch.kv_indptr,
                                           out, lse, max(batch.k_per_seq) + 1, batch.max_kv_len,
                                           1.0 / math.sqrt(wl.D))
    return out, lse


def _bits(t):
    return t.view(torch.int16 if t.element_size() == 2 else torch.int32)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_two_calls_in_a_row_match_the_workspace_entry_point(oracle, dtype):
    heads = dict(Hq=28, Hkv=4, D=128) if dtype == "bf16" else dict(Hq=4, Hkv=1, D=64)
    big = synth.Workload("static_big", B=96, k=3, V=64, dtype=dtype, len_dist="uniform", len_lo=40, len_hi=3000,
                         seed=21, **heads)
    small = synth.Workload("static_small", B=5, k=2, V=64, dtype=dtype, len_dist="uniform", len_lo=3, len_hi=400,
                           seed=22, **heads)
    b1 = synth.make_batch(big, device="cuda", with_logits=False)
    b2 = synth.make_batch(small, device="cuda", with_logits=False)
    binding.respec_static_scratch_init()
    assert binding.respec_static_scratch_bytes() == 40 << 20
    # the static calls back to back on one stream, nothing in between
    o1, l1 = _static_attention(b1)
    o2, l2 = _static_attention(b2)
    torch.cuda.synchronize()
    r1, rl1 = gpu_attention(b1)
    r2, rl2 = gpu_attention(b2)
    torch.cuda.synchronize()
    for got, ref in ((o1, r1), (o2, r2), (l1, rl1), (l2, rl2)):
        assert torch.isfinite(got.float()).all()
        assert torch.equal(_bits(got), _bits(ref))
    # and the smaller one against the oracle itself (the larger one's parity is the other entry point's)
    ref, ref_lse = oracle_attention(oracle, b2)
    tol = 2e-2 if dtype == "bf16" else 1e-5
    assert (o2.double().cpu().numpy() - ref).__abs__().max() <= tol
    assert (l2.double().cpu().numpy() - ref_lse).__abs__().max() <= (1e-3 if dtype == "bf16" else 1e-5)


def test_a_batch_whose_scratch_does_not_fit_is_refused():
    # 12 query heads per KV head x 9 rows = 108 columns: the partials of 1024 ranges need more
    # than the 40 MiB the library carries; nothing is launched
    lib = binding.load()
    x = torch.zeros(64, dtype=torch.uint8, device="cuda")
    ptr = ctypes.c_void_p(x.data_ptr())
    st = lib.respec_verify_attention_static(ptr, ptr, ptr, ptr, ptr, ptr, None, 4, 36, 4000, 9, 1000, 48, 4, 128, 0.1,
                                            binding.RESPEC_BF16, None)
    assert st == 3, lib.respec_last_error()
    assert b"built-in buffer" in lib.respec_last_error()
