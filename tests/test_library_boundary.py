"""CPU-side checks of the C boundary: the library loads, exports every symbol the header
declares, and rejects bad arguments on the host before anything touches a GPU."""
import ctypes
import os
import re

import pytest

from paper_2510_26475_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(build.LIB_PATH):
        build.build()
    return binding.load()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "respec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(respec_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_symbols()
    assert set(names) == set(binding.EXPORTED_SYMBOLS)
    for name in names:
        assert getattr(lib, name) is not None


def test_version_and_status_strings(lib):
    assert lib.respec_version() >= 100
    texts = {lib.respec_status_string(i).decode() for i in range(5)}
    assert len(texts) == 5 and "ok" in texts


def test_workspace_query(lib):
    f = lib.respec_verify_attention_workspace_bytes
    a = f(256, 1024, 668000, 4, 8192, 28, 4, 128, binding.RESPEC_BF16)
    assert a > 0 and a % 256 == 0
    assert f(256, 1024, 668000, 4, 8192, 28, 5, 128, binding.RESPEC_BF16) == 0     # Hq % Hkv
    assert f(256, 1024, 668000, 4, 8192, 28, 4, 96, binding.RESPEC_BF16) == 0      # head size
    assert f(0, 0, 0, 4, 8192, 28, 4, 128, binding.RESPEC_BF16) == 0
    w = lib.respec_rejection_sample_workspace_bytes(256, 1024, 151936, binding.RESPEC_BF16)
    assert w > 0 and w % 256 == 0                  # one mailbox per sequence
    assert lib.respec_rejection_sample_workspace_bytes(0, 0, 151936, binding.RESPEC_BF16) == 0


def test_attention_argument_errors_need_no_gpu(lib):
    null = ctypes.c_void_p(None)
    bogus = ctypes.c_void_p(0x1000)
    call = lib.respec_verify_attention
    # null pointers
    st = call(null, null, null, null, null, null, null, 1, 4, 100, 4, 100, 8, 2, 128, 0.1,
              binding.RESPEC_BF16, null, 0, null)
    assert st == 1 and b"null" in lib.respec_last_error()
    # Hq not a multiple of Hkv
    st = call(bogus, bogus, bogus, bogus, bogus, bogus, null, 1, 4, 100, 4, 100, 7, 2, 128, 0.1,
              binding.RESPEC_BF16, bogus, 1 << 30, null)
    assert st == 1
    # unsupported head size
    st = call(bogus, bogus, bogus, bogus, bogus, bogus, null, 1, 4, 100, 4, 100, 8, 2, 96, 0.1,
              binding.RESPEC_BF16, bogus, 1 << 30, null)
    assert st == 2
    # cache shorter than the new tokens
    st = call(bogus, bogus, bogus, bogus, bogus, bogus, null, 1, 4, 3, 4, 3, 8, 2, 128, 0.1,
              binding.RESPEC_BF16, bogus, 1 << 30, null)
    assert st == 1
    # misaligned q
    st = call(ctypes.c_void_p(0x1004), bogus, bogus, bogus, bogus, bogus, null, 1, 4, 100, 4, 100,
              8, 2, 128, 0.1, binding.RESPEC_BF16, bogus, 1 << 30, null)
    assert st == 1 and b"aligned" in lib.respec_last_error()
    # workspace too small
    st = call(bogus, bogus, bogus, bogus, bogus, bogus, null, 1, 4, 100, 4, 100, 8, 2, 128, 0.1,
              binding.RESPEC_BF16, bogus, 16, null)
    assert st == 3


def test_sampler_argument_errors_need_no_gpu(lib):
    null = ctypes.c_void_p(None)
    bogus = ctypes.c_void_p(0x1000)
    call = lib.respec_rejection_sample

    def run(**kw):
        a = dict(t=bogus, d=bogus, tok=bogus, qi=bogus, ua=bogus, uf=bogus, ot=bogus, on=bogus,
                 of=null, B=2, total_q=8, max_k=3, V=1024, ld_t=1024, ld_d=1024, T=1.0,
                 dt=binding.RESPEC_F32)
        a.update(kw)
        return call(a["t"], a["d"], a["tok"], a["qi"], a["ua"], a["uf"], a["ot"], a["on"], a["of"],
                    a["B"], a["total_q"], a["max_k"], a["V"], a["ld_t"], a["ld_d"], a["T"], a["dt"],
                    null, 0, null)

    assert run(T=0.0) == 1
    assert run(T=-1.0) == 1
    assert run(T=float("nan")) == 1
    assert run(t=null) == 1
    assert run(d=null) == 1                  # drafts present but no drafter logits
    assert run(ld_t=1000) == 1               # stride below V
    assert run(max_k=2) == 1                 # 2 sequences * 2 < 6 drafted tokens
    assert run(V=0) == 1
    assert run(dt=7) == 1
    assert run(B=0) == 1


def test_tree_entry_points_argument_errors_need_no_gpu(lib):
    null = ctypes.c_void_p(None)
    bogus = ctypes.c_void_p(0x1000)
    attn = lib.respec_verify_attention_tree
    # more rows per sequence than the mask has bits
    st = attn(bogus, bogus, bogus, bogus, bogus, bogus, bogus, null, 1, 65, 100, 65, 100, 8, 2, 128, 0.1,
              binding.RESPEC_BF16, bogus, 1 << 30, null)
    assert st == 2
    # no mask
    st = attn(bogus, bogus, bogus, bogus, bogus, null, bogus, null, 1, 4, 100, 4, 100, 8, 2, 128, 0.1,
              binding.RESPEC_BF16, bogus, 1 << 30, null)
    assert st == 1
    call = lib.respec_tree_rejection_sample

    def run(**kw):
        a = dict(t=bogus, d=bogus, tok=bogus, par=bogus, qi=bogus, ua=bogus, uf=bogus, ot=bogus, op=bogus,
                 on=bogus, of=null, B=2, total_q=8, max_rows=4, max_depth=3, V=1024, ld_t=1024, ld_d=1024,
                 T=1.0, dt=binding.RESPEC_F32)
        a.update(kw)
        return call(a["t"], a["d"], a["tok"], a["par"], a["qi"], a["ua"], a["uf"], a["ot"], a["op"], a["on"],
                    a["of"], a["B"], a["total_q"], a["max_rows"], a["max_depth"], a["V"], a["ld_t"], a["ld_d"],
                    a["T"], a["dt"], null)

    assert run(T=0.0) == 1
    assert run(T=float("inf")) == 1
    assert run(d=null) == 1
    assert run(par=null) == 1
    assert run(op=null) == 1
    assert run(ld_d=1000) == 1
    assert run(max_rows=3) == 1              # 2 sequences * 3 rows < 8 rows
    assert run(max_rows=65, total_q=100) == 2
    assert run(max_depth=-1) == 1
    assert run(dt=7) == 1
