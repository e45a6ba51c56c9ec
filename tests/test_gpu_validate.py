"""respec_validate_batch: the debug check of device-side index arrays and drafted tokens."""
import pytest
import torch

from paper_2510_26475_amd import binding, synth

pytestmark = pytest.mark.gpu


def _batch():
    wl = synth.Workload("val", B=0, k=0, Hq=4, Hkv=1, D=64, V=1000, dtype="f32", len_dist="uniform",
                        len_lo=1, len_hi=1)
    ks = [3, 0, 2, 4, 1, 4, 0, 2]
    return synth.make_batch(wl, device="cuda", kv_lens=[10 + 7 * i for i in range(len(ks))], k_per_seq=ks, seed=1)


def _validate(b, q_indptr=None, kv_indptr=None, tokens=None, max_q=None, max_kv=None, total_q=None, total_kv=None):
    binding.respec_validate_batch(b.q_indptr if q_indptr is None else q_indptr,
                                  b.kv_indptr if kv_indptr is None else kv_indptr,
                                  b.draft_tokens if tokens is None else tokens,
                                  b.total_q if total_q is None else total_q,
                                  b.total_kv if total_kv is None else total_kv,
                                  b.max_k + 1 if max_q is None else max_q,
                                  b.max_kv_len if max_kv is None else max_kv, b.wl.V)


def test_a_good_batch_passes():
    b = _batch()
    _validate(b)
    binding.respec_validate_batch(b.q_indptr, None, None, b.total_q, 0, b.max_k + 1, 0, b.wl.V)   # paged form


@pytest.mark.parametrize("case,seq,text", [
    ("token_high", 3, "drafted token"), ("token_negative", 0, "drafted token"),
    ("rows_too_many", 3, "number of rows"), ("rows_zero", 4, "number of rows"),
    ("short_cache", 2, "cached length"), ("long_cache", 7, "cached length"),
    ("bad_start", 0, "start at 0"), ("bad_total", 7, "last entry"),
])
def test_defects_are_reported_with_their_sequence(case, seq, text):
    b = _batch()
    qi, ki, tok = b.q_indptr.clone(), b.kv_indptr.clone(), b.draft_tokens.clone()
    kw = {}
    if case == "token_high":
        tok[int(qi[3]) - 3 + 1] = b.wl.V
    elif case == "token_negative":
        tok[0] = -1
    elif case == "rows_too_many":
        kw["max_q"] = 4                        # sequence 3 has five rows
    elif case == "rows_zero":
        qi[5:] -= 2                            # sequence 4 (two rows) is left with none
        kw["total_q"] = b.total_q - 2
        tok = tok[:-2].contiguous()
    elif case == "short_cache":
        ki[3:] -= int(ki[3] - ki[2]) - 1       # sequence 2 keeps one cached token for three rows
        kw["total_kv"] = int(ki[-1])
    elif case == "long_cache":
        kw["max_kv"] = b.max_kv_len - 1        # the last sequence is the longest
    elif case == "bad_start":
        qi[0] = 1
    elif case == "bad_total":
        kw["total_kv"] = b.total_kv + 1
    with pytest.raises(binding.RespecError) as e:
        _validate(b, q_indptr=qi, kv_indptr=ki, tokens=tok, **kw)
    assert e.value.status == 1 and f"sequence {seq}:" in str(e.value) and text in str(e.value), str(e.value)


def test_the_lowest_bad_sequence_is_named():
    b = _batch()
    tok = b.draft_tokens.clone()
    tok[-1] = 10 ** 6
    tok[0] = 10 ** 6
    with pytest.raises(binding.RespecError) as e:
        _validate(b, tokens=tok)
    assert "sequence 0:" in str(e.value)


def test_host_side_argument_errors():
    b = _batch()
    lib = binding.load()
    assert lib.respec_validate_batch(b.q_indptr.data_ptr(), None, None, 8, b.total_q, 0, 5, 0, 1000, None, 0, None) == 3
    assert lib.respec_validate_batch(None, None, None, 8, b.total_q, 0, 5, 0, 1000, None, 0, None) == 1
    assert lib.respec_validate_batch_workspace_bytes(0) == 0
