"""CPU oracle for the speculative-decoding verify step -- TEST INFRASTRUCTURE ONLY.

A thin ctypes loader around ``respec_oracle.c`` (plain C, fp64).  Only the tests,
``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may import this
package; the product (``paper_2510_26475_amd``) never does and the two share no code.

Arrays are numpy, host side.  bf16 data is passed as ``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "respec_oracle.c")
_LIB = os.path.join(_HERE, "librespec_oracle.so")
# A test may point the loader at another build of the same source (the sanitizer build of
# tests/test_oracle_sanitizers.py); that build is then used as it is.
_OVERRIDE = os.environ.get("RESPEC_ORACLE_LIBRARY")

F32 = 0
BF16 = 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no HIP, no third-party code)."""
    global _LIB
    if _OVERRIDE:
        _LIB = _OVERRIDE
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c = ctypes
        lib.respec_oracle_verify_attention.restype = c.c_int
        lib.respec_oracle_verify_attention.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
            c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_double, c.c_int, c.c_int]
        lib.respec_oracle_rejection_sample.restype = c.c_int
        lib.respec_oracle_rejection_sample.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
            c.c_void_p, c.c_void_p, c.c_void_p,
            c.c_int32, c.c_int32, c.c_int32, c.c_int64, c.c_int64, c.c_double, c.c_int, c.c_int]
        lib.respec_oracle_rejection_sample_per_seq.restype = c.c_int
        lib.respec_oracle_rejection_sample_per_seq.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
            c.c_void_p, c.c_void_p, c.c_void_p,
            c.c_int32, c.c_int32, c.c_int32, c.c_int64, c.c_int64, c.c_int, c.c_int]
        lib.respec_oracle_verify_attention_tree.restype = c.c_int
        lib.respec_oracle_verify_attention_tree.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
            c.c_void_p, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_double, c.c_int, c.c_int]
        lib.respec_oracle_tree_rejection_sample.restype = c.c_int
        lib.respec_oracle_tree_rejection_sample.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
            c.c_int32, c.c_int32, c.c_int32, c.c_int64, c.c_int64, c.c_double, c.c_int, c.c_int]
        lib.respec_oracle_verify_attention_paged.restype = c.c_int
        lib.respec_oracle_verify_attention_paged.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
            c.c_void_p, c.c_void_p, c.c_void_p,
            c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_double, c.c_int, c.c_int]
        lib.respec_oracle_commit_accepted_paged.restype = c.c_int
        lib.respec_oracle_commit_accepted_paged.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
            c.c_int32, c.c_void_p, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int]
        lib.respec_oracle_kd_rows.restype = c.c_int
        lib.respec_oracle_kd_rows.argtypes = [
            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
            c.c_int32, c.c_int32, c.c_int64, c.c_int64, c.c_int, c.c_int]
        lib.respec_oracle_softmax_rows.restype = c.c_int
        lib.respec_oracle_softmax_rows.argtypes = [
            c.c_void_p, c.c_int32, c.c_int32, c.c_int64, c.c_double, c.c_int, c.c_void_p]
        lib.respec_oracle_max_threads.restype = c.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().respec_oracle_max_threads())


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check_elems(a: np.ndarray, dtype: int, name: str) -> np.ndarray:
    want = np.float32 if dtype == F32 else np.uint16
    if a.dtype != want:
        raise TypeError(f"{name}: expected {want.__name__} for dtype code {dtype}, got {a.dtype}")
    return np.ascontiguousarray(a)


def verify_attention(q, k_cache, v_cache, q_indptr, kv_indptr, Hq, Hkv, D, sm_scale, dtype,
                     want_lse=False, n_threads=1):
    """q [total_q,Hq,D], k_cache/v_cache [total_kv,Hkv,D] (float32 or uint16 bf16 bits).

    Returns out [total_q,Hq,D] float64 (and lse [total_q,Hq] float64 when asked).
    """
    q = _check_elems(q, dtype, "q")
    k_cache = _check_elems(k_cache, dtype, "k_cache")
    v_cache = _check_elems(v_cache, dtype, "v_cache")
    q_indptr = np.ascontiguousarray(q_indptr, dtype=np.int32)
    kv_indptr = np.ascontiguousarray(kv_indptr, dtype=np.int64)
    B = q_indptr.shape[0] - 1
    total_q = int(q_indptr[-1])
    total_kv = int(kv_indptr[-1])
    assert q.size == total_q * Hq * D, "q size does not match q_indptr"
    assert k_cache.size == total_kv * Hkv * D and v_cache.size == total_kv * Hkv * D
    out = np.zeros((total_q, Hq, D), dtype=np.float64)
    lse = np.zeros((total_q, Hq), dtype=np.float64) if want_lse else None
    rc = _load().respec_oracle_verify_attention(
        _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(q_indptr), _ptr(kv_indptr), _ptr(out),
        _ptr(lse), B, Hq, Hkv, D, float(sm_scale), dtype, n_threads)
    if rc != 0:
        raise RuntimeError(f"respec_oracle_verify_attention failed with code {rc}")
    return (out, lse) if want_lse else out


def verify_attention_tree(q, k_cache, v_cache, q_indptr, kv_indptr, tree_mask, Hq, Hkv, D, sm_scale,
                          dtype, want_lse=False, n_threads=1):
    """As verify_attention, with tree_mask [total_q] uint64: bit j of row i's word says that the
    sequence's j-th new token is visible to row i (its ancestors and itself)."""
    q = _check_elems(q, dtype, "q")
    k_cache = _check_elems(k_cache, dtype, "k_cache")
    v_cache = _check_elems(v_cache, dtype, "v_cache")
    q_indptr = np.ascontiguousarray(q_indptr, dtype=np.int32)
    kv_indptr = np.ascontiguousarray(kv_indptr, dtype=np.int64)
    tree_mask = np.ascontiguousarray(tree_mask, dtype=np.uint64)
    B = q_indptr.shape[0] - 1
    total_q = int(q_indptr[-1])
    assert tree_mask.shape == (total_q,)
    out = np.zeros((total_q, Hq, D), dtype=np.float64)
    lse = np.zeros((total_q, Hq), dtype=np.float64) if want_lse else None
    rc = _load().respec_oracle_verify_attention_tree(
        _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(q_indptr), _ptr(kv_indptr), _ptr(tree_mask),
        _ptr(out), _ptr(lse), B, Hq, Hkv, D, float(sm_scale), dtype, n_threads)
    if rc != 0:
        raise RuntimeError(f"respec_oracle_verify_attention_tree failed with code {rc}")
    return (out, lse) if want_lse else out


def verify_attention_paged(q, k_pages, v_pages, q_indptr, page_indptr, page_table, kv_len, Hq, Hkv, D,
                           sm_scale, dtype, tree_mask=None, want_lse=False, n_threads=1):
    """k_pages, v_pages [num_pages, page_size, Hkv, D]; sequence b owns the pages
    page_table[page_indptr[b]:page_indptr[b+1]] in token order and holds kv_len[b] tokens."""
    q = _check_elems(q, dtype, "q")
    k_pages = _check_elems(k_pages, dtype, "k_pages")
    v_pages = _check_elems(v_pages, dtype, "v_pages")
    assert k_pages.ndim == 4 and k_pages.shape == v_pages.shape and k_pages.shape[2:] == (Hkv, D)
    num_pages, page_size = k_pages.shape[:2]
    q_indptr = np.ascontiguousarray(q_indptr, dtype=np.int32)
    page_indptr = np.ascontiguousarray(page_indptr, dtype=np.int32)
    page_table = np.ascontiguousarray(page_table, dtype=np.int32)
    kv_len = np.ascontiguousarray(kv_len, dtype=np.int32)
    B = q_indptr.shape[0] - 1
    total_q = int(q_indptr[-1])
    assert page_indptr.shape == (B + 1,) and kv_len.shape == (B,) and page_table.shape[0] >= int(page_indptr[-1])
    if tree_mask is not None:
        tree_mask = np.ascontiguousarray(tree_mask, dtype=np.uint64)
        assert tree_mask.shape == (total_q,)
    out = np.zeros((total_q, Hq, D), dtype=np.float64)
    lse = np.zeros((total_q, Hq), dtype=np.float64) if want_lse else None
    rc = _load().respec_oracle_verify_attention_paged(
        _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(q_indptr), _ptr(page_indptr), _ptr(page_table),
        _ptr(kv_len), _ptr(tree_mask), _ptr(out), _ptr(lse), B, num_pages, page_size, Hq, Hkv, D,
        float(sm_scale), dtype, n_threads)
    if rc != 0:
        raise RuntimeError(f"respec_oracle_verify_attention_paged failed with code {rc}")
    return (out, lse) if want_lse else out


def commit_accepted_paged(k_pages, v_pages, q_indptr, page_indptr, page_table, kv_len, num_accepted, dtype,
                          path=None):
    """Moves the K/V of the accepted rows behind the last committed token and cuts the lengths.
    k_pages, v_pages and kv_len are changed IN PLACE (they must be C-contiguous arrays of the right type)."""
    want = np.float32 if dtype == F32 else np.uint16
    for a, name in ((k_pages, "k_pages"), (v_pages, "v_pages")):
        if a.dtype != want or not a.flags["C_CONTIGUOUS"]:
            raise TypeError(f"{name} must be a C-contiguous {want.__name__} array")
    if kv_len.dtype != np.int32 or not kv_len.flags["C_CONTIGUOUS"]:
        raise TypeError("kv_len must be a C-contiguous int32 array")
    num_pages, page_size, Hkv, D = k_pages.shape
    q_indptr = np.ascontiguousarray(q_indptr, dtype=np.int32)
    page_indptr = np.ascontiguousarray(page_indptr, dtype=np.int32)
    page_table = np.ascontiguousarray(page_table, dtype=np.int32)
    num_accepted = np.ascontiguousarray(num_accepted, dtype=np.int32)
    B = q_indptr.shape[0] - 1
    stride = 0
    if path is not None:
        path = np.ascontiguousarray(path, dtype=np.int32)
        assert path.ndim == 2 and path.shape[0] == B
        stride = path.shape[1]
    rc = _load().respec_oracle_commit_accepted_paged(
        _ptr(k_pages), _ptr(v_pages), _ptr(q_indptr), _ptr(page_indptr), _ptr(page_table), _ptr(kv_len),
        _ptr(path), stride, _ptr(num_accepted), B, num_pages, page_size, Hkv, D, dtype)
    if rc != 0:
        raise RuntimeError(f"respec_oracle_commit_accepted_paged failed with code {rc}")


def kd_rows(target_logits, draft_logits, row_weight, dtype, n_threads=1):
    """Reward-weighted KD per logits row: returns (grad [rows,V] float64 = w (q - p),
    row_loss [rows] float64 = w KL(p||q), total float)."""
    target_logits = _check_elems(target_logits, dtype, "target_logits")
    draft_logits = _check_elems(draft_logits, dtype, "draft_logits")
    rows, V = target_logits.shape
    assert draft_logits.shape == (rows, V)
    row_weight = np.ascontiguousarray(row_weight, dtype=np.float32)
    assert row_weight.shape == (rows,)
    grad = np.empty((rows, V), dtype=np.float64)
    row_loss = np.empty((rows,), dtype=np.float64)
    total = np.zeros((1,), dtype=np.float64)
    rc = _load().respec_oracle_kd_rows(_ptr(target_logits), _ptr(draft_logits), _ptr(row_weight), _ptr(grad),
                                       _ptr(row_loss), _ptr(total), rows, V, V, V, dtype, n_threads)
    if rc != 0:
        raise RuntimeError(f"respec_oracle_kd_rows failed with code {rc}")
    return grad, row_loss, float(total[0])


def tree_rejection_sample(target_logits, draft_logits, node_tokens, parent, q_indptr, u_accept,
                          u_final, max_depth, temperature, dtype, n_threads=1):
    """target_logits, draft_logits [total_q,V]; node_tokens, parent, u_accept [total_q].

    Returns (out_tokens [B,max_depth+1], out_path [B,max(max_depth,1)], num_accepted [B], flags [B]).
    """
    target_logits = _check_elems(target_logits, dtype, "target_logits")
    draft_logits = _check_elems(draft_logits, dtype, "draft_logits")
    q_indptr = np.ascontiguousarray(q_indptr, dtype=np.int32)
    B = q_indptr.shape[0] - 1
    total_q, V = target_logits.shape
    assert total_q == int(q_indptr[-1]) and draft_logits.shape == (total_q, V)
    node_tokens = np.ascontiguousarray(node_tokens, dtype=np.int32)
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    u_accept = np.ascontiguousarray(u_accept, dtype=np.float32)
    u_final = np.ascontiguousarray(u_final, dtype=np.float32)
    assert node_tokens.shape == parent.shape == u_accept.shape == (total_q,) and u_final.shape == (B,)
    out_tokens = np.empty((B, max_depth + 1), dtype=np.int32)
    out_path = np.empty((B, max(max_depth, 1)), dtype=np.int32)
    num_accepted = np.empty((B,), dtype=np.int32)
    flags = np.empty((B,), dtype=np.int32)
    rc = _load().respec_oracle_tree_rejection_sample(
        _ptr(target_logits), _ptr(draft_logits), _ptr(node_tokens), _ptr(parent), _ptr(q_indptr),
        _ptr(u_accept), _ptr(u_final), _ptr(out_tokens), _ptr(out_path), _ptr(num_accepted),
        _ptr(flags), B, max_depth, V, V, V, float(np.float32(temperature)), dtype, n_threads)
    if rc != 0:
        raise RuntimeError(f"respec_oracle_tree_rejection_sample failed with code {rc}")
    return out_tokens, out_path, num_accepted, flags


def rejection_sample(target_logits, draft_logits, draft_tokens, q_indptr, u_accept, u_final,
                     max_k, temperature, dtype, n_threads=1):
    """target_logits [total_q,V], draft_logits [total_q-B,V] (float32 or uint16 bf16 bits).

    The temperature is rounded to binary32 first: the boundary passes it as a C float.
    Returns (out_tokens [B,max_k+1] int32, num_accepted [B] int32, flags [B] int32).
    """
    target_logits = _check_elems(target_logits, dtype, "target_logits")
    q_indptr = np.ascontiguousarray(q_indptr, dtype=np.int32)
    B = q_indptr.shape[0] - 1
    V = target_logits.shape[-1]
    assert target_logits.ndim == 2 and target_logits.shape[0] == int(q_indptr[-1])
    n_draft = int(q_indptr[-1]) - B
    if n_draft > 0:
        draft_logits = _check_elems(draft_logits, dtype, "draft_logits")
        assert draft_logits.shape == (n_draft, V)
        draft_tokens = np.ascontiguousarray(draft_tokens, dtype=np.int32)
        u_accept = np.ascontiguousarray(u_accept, dtype=np.float32)
        assert draft_tokens.shape == (n_draft,) and u_accept.shape == (n_draft,)
    else:
        draft_logits = draft_tokens = u_accept = None
    u_final = np.ascontiguousarray(u_final, dtype=np.float32)
    assert u_final.shape == (B,)
    out_tokens = np.empty((B, max_k + 1), dtype=np.int32)
    num_accepted = np.empty((B,), dtype=np.int32)
    flags = np.empty((B,), dtype=np.int32)
    rc = _load().respec_oracle_rejection_sample(
        _ptr(target_logits), _ptr(draft_logits), _ptr(draft_tokens), _ptr(q_indptr),
        _ptr(u_accept), _ptr(u_final), _ptr(out_tokens), _ptr(num_accepted), _ptr(flags),
        B, max_k, V, V, V, float(np.float32(temperature)), dtype, n_threads)
    if rc != 0:
        raise RuntimeError(f"respec_oracle_rejection_sample failed with code {rc}")
    return out_tokens, num_accepted, flags


def rejection_sample_per_seq(target_logits, draft_logits, draft_tokens, q_indptr, u_accept, u_final,
                             max_k, temperatures, dtype, n_threads=1):
    """As ``rejection_sample`` with one binary32 temperature per sequence; 0 selects greedy
    verification (accept iff the drafted token is the target row's first argmax)."""
    target_logits = _check_elems(target_logits, dtype, "target_logits")
    q_indptr = np.ascontiguousarray(q_indptr, dtype=np.int32)
    B = q_indptr.shape[0] - 1
    V = target_logits.shape[-1]
    assert target_logits.ndim == 2 and target_logits.shape[0] == int(q_indptr[-1])
    n_draft = int(q_indptr[-1]) - B
    if n_draft > 0:
        draft_tokens = np.ascontiguousarray(draft_tokens, dtype=np.int32)
        assert draft_tokens.shape == (n_draft,)
        if draft_logits is not None:
            draft_logits = _check_elems(draft_logits, dtype, "draft_logits")
            assert draft_logits.shape == (n_draft, V)
        if u_accept is not None:
            u_accept = np.ascontiguousarray(u_accept, dtype=np.float32)
            assert u_accept.shape == (n_draft,)
    else:
        draft_logits = draft_tokens = u_accept = None
    u_final = np.ascontiguousarray(u_final, dtype=np.float32)
    temperatures = np.ascontiguousarray(temperatures, dtype=np.float32)
    assert u_final.shape == (B,) and temperatures.shape == (B,)
    out_tokens = np.empty((B, max_k + 1), dtype=np.int32)
    num_accepted = np.empty((B,), dtype=np.int32)
    flags = np.empty((B,), dtype=np.int32)
    rc = _load().respec_oracle_rejection_sample_per_seq(
        _ptr(target_logits), _ptr(draft_logits), _ptr(draft_tokens), _ptr(q_indptr), _ptr(u_accept),
        _ptr(u_final), _ptr(temperatures), _ptr(out_tokens), _ptr(num_accepted), _ptr(flags),
        B, max_k, V, V, V, dtype, n_threads)
    if rc != 0:
        raise RuntimeError(f"respec_oracle_rejection_sample_per_seq failed with code {rc}")
    return out_tokens, num_accepted, flags


def softmax_rows(logits, temperature, dtype):
    """softmax(logits/T) row by row in fp64, as the sampler oracle computes it."""
    logits = _check_elems(logits, dtype, "logits")
    n, V = logits.shape
    out = np.empty((n, V), dtype=np.float64)
    rc = _load().respec_oracle_softmax_rows(_ptr(logits), n, V, V, float(np.float32(temperature)), dtype,
                                            _ptr(out))
    if rc != 0:
        raise RuntimeError(f"respec_oracle_softmax_rows failed with code {rc}")
    return out


def solver_pick(points, active_batch, draft_us_fixed, draft_us_per_seq):
    """The Solver's choice of the draft length for one active batch size, from a profile table
    (Section 5.2, "Solver: Offline Profiling Guided Search") under the cost model of Eq. 4.

    ``points``: iterable of (batch, k, step_us, emitted_per_seq) measured offline; k = 0 is plain
    decoding.  For every k in the table the step time and the emitted tokens per sequence at
    ``active_batch`` are interpolated linearly between the profiled batch sizes (end values
    outside their range).  Eq. 4's cost per produced token, with the measured quantities in the
    place of its symbols: (k * C_q + k * C_p / alpha) / (r * k)  ->
    (k * draft_us + step_us_k) / emitted_k, draft_us = draft_us_fixed + draft_us_per_seq * batch.
    Returns (best_k, speedup over k = 0, cost of best_k, {k: cost}); ties go to the smaller k.
    Plain Python, for small tables.
    """
    by_k = {}
    for (B, k, t, e) in points:
        by_k.setdefault(int(k), []).append((float(B), float(t), float(e)))
    if 0 not in by_k:
        raise ValueError("the profile needs the plain-decoding points (k = 0)")
    b = float(active_batch)
    draft = float(draft_us_fixed) + float(draft_us_per_seq) * b

    def interp(rows, col):
        rows = sorted(rows)
        if b <= rows[0][0]:
            return rows[0][col]
        if b >= rows[-1][0]:
            return rows[-1][col]
        for lo, hi in zip(rows[:-1], rows[1:]):
            if lo[0] <= b <= hi[0]:
                if hi[0] == lo[0]:
                    return lo[col]
                w = (b - lo[0]) / (hi[0] - lo[0])
                return lo[col] + w * (hi[col] - lo[col])
        raise AssertionError

    cost = {}
    for k, rows in by_k.items():
        t, e = interp(rows, 1), interp(rows, 2)
        cost[k] = (k * draft + t) / e
    best = min(sorted(cost), key=lambda k: (cost[k], k))
    return best, cost[0] / cost[best], cost[best], cost
