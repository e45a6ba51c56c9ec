"""ctypes binding of librespec.so: argument marshalling only.

Same names as the C boundary (``include/respec.h``).  Torch tensors are used for device
memory and the current stream; every step of the verify path runs in the HIP kernels.
There is no CPU fallback: a missing library or a non-CUDA tensor is an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from . import build as _build

RESPEC_F32 = 0
RESPEC_BF16 = 1

_lib = None


class RespecError(RuntimeError):
    def __init__(self, status: int, text: str, detail: str):
        super().__init__(f"librespec status {status} ({text}): {detail}")
        self.status = status


def library_path() -> str:
    """Path of librespec.so; RESPEC_LIBRARY_PATH points at another build of it (experiments)."""
    return os.environ.get("RESPEC_LIBRARY_PATH") or _build.LIB_PATH


def load():
    """Load librespec.so (building it first only if it has never been built)."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        _build.build()
    if not os.path.exists(path):
        raise RuntimeError(f"librespec.so not found at {path}; run python -m paper_2510_26475_amd.build")
    lib = ctypes.CDLL(path)
    c = ctypes
    lib.respec_status_string.restype = c.c_char_p
    lib.respec_status_string.argtypes = [c.c_int]
    lib.respec_last_error.restype = c.c_char_p
    lib.respec_last_error.argtypes = []
    lib.respec_version.restype = c.c_int
    lib.respec_version.argtypes = []
    lib.respec_verify_attention_workspace_bytes.restype = c.c_size_t
    lib.respec_verify_attention_workspace_bytes.argtypes = [
        c.c_int32, c.c_int32, c.c_int64, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32,
        c.c_int]
    lib.respec_verify_attention.restype = c.c_int
    lib.respec_verify_attention.argtypes = [
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_int32, c.c_int32, c.c_int64, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32,
        c.c_float, c.c_int, c.c_void_p, c.c_size_t, c.c_void_p]
    lib.respec_verify_attention_tree.restype = c.c_int
    lib.respec_verify_attention_tree.argtypes = [
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_int32, c.c_int32, c.c_int64, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32,
        c.c_float, c.c_int, c.c_void_p, c.c_size_t, c.c_void_p]
    lib.respec_verify_attention_next_layer.restype = c.c_int
    lib.respec_verify_attention_next_layer.argtypes = lib.respec_verify_attention_tree.argtypes
    lib.respec_static_scratch_bytes.restype = c.c_size_t
    lib.respec_static_scratch_bytes.argtypes = []
    lib.respec_static_scratch_init.restype = c.c_int
    lib.respec_static_scratch_init.argtypes = []
    lib.respec_verify_attention_static.restype = c.c_int
    lib.respec_verify_attention_static.argtypes = [
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_int32, c.c_int32, c.c_int64, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32,
        c.c_float, c.c_int, c.c_void_p]
    lib.respec_reload_knobs.restype = None
    lib.respec_reload_knobs.argtypes = []
    lib.respec_profile_mark_main.restype = None
    lib.respec_profile_mark_main.argtypes = [c.c_void_p, c.c_void_p]
    lib.respec_rejection_sample_workspace_bytes.restype = c.c_size_t
    lib.respec_rejection_sample_workspace_bytes.argtypes = [c.c_int32, c.c_int32, c.c_int32, c.c_int]
    lib.respec_rejection_sample.restype = c.c_int
    lib.respec_rejection_sample.argtypes = [
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int64, c.c_int64,
        c.c_float, c.c_int, c.c_void_p, c.c_size_t, c.c_void_p]
    lib.respec_rejection_sample_per_seq.restype = c.c_int
    lib.respec_rejection_sample_per_seq.argtypes = [
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int64, c.c_int64, c.c_int, c.c_void_p]
    lib.respec_tree_rejection_sample.restype = c.c_int
    lib.respec_tree_rejection_sample.argtypes = [
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int64, c.c_int64,
        c.c_float, c.c_int, c.c_void_p]
    lib.respec_verify_attention_paged.restype = c.c_int
    lib.respec_verify_attention_paged.argtypes = [
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_void_p, c.c_void_p,
        c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32,
        c.c_int32, c.c_float, c.c_int, c.c_void_p, c.c_size_t, c.c_void_p]
    lib.respec_verify_attention_paged_next_layer.restype = c.c_int
    lib.respec_verify_attention_paged_next_layer.argtypes = lib.respec_verify_attention_paged.argtypes
    lib.respec_commit_accepted_paged.restype = c.c_int
    lib.respec_commit_accepted_paged.argtypes = [
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32,
        c.c_void_p, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32, c.c_int32,
        c.c_int, c.c_void_p]
    lib.respec_kd_rows_workspace_bytes.restype = c.c_size_t
    lib.respec_kd_rows_workspace_bytes.argtypes = [c.c_int32, c.c_int32, c.c_int]
    lib.respec_kd_rows.restype = c.c_int
    lib.respec_kd_rows.argtypes = [
        c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p,
        c.c_int32, c.c_int32, c.c_int64, c.c_int64, c.c_int64, c.c_int, c.c_void_p, c.c_size_t, c.c_void_p]
    lib.respec_validate_batch_workspace_bytes.restype = c.c_size_t
    lib.respec_validate_batch_workspace_bytes.argtypes = [c.c_int32]
    lib.respec_validate_batch.restype = c.c_int
    lib.respec_validate_batch.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32, c.c_int64,
                                          c.c_int32, c.c_int32, c.c_int32, c.c_void_p, c.c_size_t, c.c_void_p]
    lib.respec_solver_pick.restype = c.c_int
    lib.respec_solver_pick.argtypes = [c.c_void_p, c.c_int32, c.c_int32, c.c_double, c.c_double,
                                       c.POINTER(c.c_int32), c.POINTER(c.c_double), c.POINTER(c.c_double)]
    _lib = lib
    return lib


class ProfilePoint(ctypes.Structure):
    """respec_profile_point_t"""
    _fields_ = [("batch", ctypes.c_int32), ("k", ctypes.c_int32), ("step_us", ctypes.c_double),
                ("emitted_per_seq", ctypes.c_double)]


EXPORTED_SYMBOLS = [
    "respec_status_string", "respec_last_error", "respec_version",
    "respec_verify_attention_workspace_bytes", "respec_verify_attention", "respec_verify_attention_tree",
    "respec_verify_attention_next_layer", "respec_verify_attention_paged_next_layer",
    "respec_rejection_sample_workspace_bytes", "respec_rejection_sample", "respec_rejection_sample_per_seq",
    "respec_tree_rejection_sample", "respec_verify_attention_paged", "respec_commit_accepted_paged",
    "respec_kd_rows_workspace_bytes", "respec_kd_rows", "respec_solver_pick",
    "respec_validate_batch_workspace_bytes", "respec_validate_batch",
    "respec_profile_mark_main",
    "respec_static_scratch_bytes", "respec_static_scratch_init", "respec_verify_attention_static",
    "respec_reload_knobs",
]


def _check(status: int):
    if status != 0:
        lib = load()
        raise RespecError(status, lib.respec_status_string(status).decode(),
                          lib.respec_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return RESPEC_F32
    if t.dtype == torch.bfloat16:
        return RESPEC_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev_ptr(t: Optional[torch.Tensor], name: str):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU (got {t.device})")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream: Optional[torch.cuda.Stream]):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def respec_reload_knobs():
    """Have the library read its RESPEC_* environment knobs again (tests and sweeps)."""
    load().respec_reload_knobs()


def respec_version() -> int:
    return int(load().respec_version())


def respec_verify_attention_workspace_bytes(B, total_q, total_kv, max_q_per_seq, max_kv_len, Hq,
                                            Hkv, D, dt) -> int:
    return int(load().respec_verify_attention_workspace_bytes(
        B, total_q, total_kv, max_q_per_seq, max_kv_len, Hq, Hkv, D, dt))


def respec_verify_attention(q, k_cache, v_cache, q_indptr, kv_indptr, out, lse, max_q_per_seq,
                            max_kv_len, sm_scale, workspace, stream=None):
    """q/out [total_q,Hq,D], k_cache/v_cache [total_kv,Hkv,D], q_indptr int32, kv_indptr int64."""
    lib = load()
    total_q, Hq, D = q.shape
    total_kv, Hkv, _ = k_cache.shape
    B = q_indptr.numel() - 1
    if q_indptr.dtype != torch.int32 or kv_indptr.dtype != torch.int64:
        raise TypeError("q_indptr must be int32 and kv_indptr int64")
    if lse is not None and lse.dtype != torch.float32:
        raise TypeError("lse must be float32")
    if out.dtype != q.dtype or k_cache.dtype != q.dtype or v_cache.dtype != q.dtype:
        raise TypeError("q, k_cache, v_cache and out must share one dtype")
    ws_ptr = _dev_ptr(workspace, "workspace") if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.respec_verify_attention(
        _dev_ptr(q, "q"), _dev_ptr(k_cache, "k_cache"), _dev_ptr(v_cache, "v_cache"),
        _dev_ptr(q_indptr, "q_indptr"), _dev_ptr(kv_indptr, "kv_indptr"), _dev_ptr(out, "out"),
        _dev_ptr(lse, "lse"), B, total_q, total_kv, max_q_per_seq, max_kv_len, Hq, Hkv, D,
        float(sm_scale), _dtype_code(q), ws_ptr, ws_bytes, _stream_ptr(stream)))


def respec_static_scratch_bytes() -> int:
    return int(load().respec_static_scratch_bytes())


def respec_static_scratch_init():
    _check(load().respec_static_scratch_init())


def respec_verify_attention_static(q, k_cache, v_cache, q_indptr, kv_indptr, out, lse, max_q_per_seq,
                                   max_kv_len, sm_scale, stream=None):
    """respec_verify_attention without a workspace: the scratch is the library's built-in buffer."""
    lib = load()
    total_q, Hq, D = q.shape
    total_kv, Hkv, _ = k_cache.shape
    B = q_indptr.numel() - 1
    if q_indptr.dtype != torch.int32 or kv_indptr.dtype != torch.int64:
        raise TypeError("q_indptr must be int32 and kv_indptr int64")
    if lse is not None and lse.dtype != torch.float32:
        raise TypeError("lse must be float32")
    if out.dtype != q.dtype or k_cache.dtype != q.dtype or v_cache.dtype != q.dtype:
        raise TypeError("q, k_cache, v_cache and out must share one dtype")
    _check(lib.respec_verify_attention_static(
        _dev_ptr(q, "q"), _dev_ptr(k_cache, "k_cache"), _dev_ptr(v_cache, "v_cache"),
        _dev_ptr(q_indptr, "q_indptr"), _dev_ptr(kv_indptr, "kv_indptr"), _dev_ptr(out, "out"),
        _dev_ptr(lse, "lse"), B, total_q, total_kv, max_q_per_seq, max_kv_len, Hq, Hkv, D,
        float(sm_scale), _dtype_code(q), _stream_ptr(stream)))


def respec_verify_attention_next_layer(q, k_cache, v_cache, q_indptr, kv_indptr, out, lse, max_q_per_seq,
                                       max_kv_len, sm_scale, workspace, tree_mask=None, stream=None):
    """Another layer of the same forward: same index arrays and sizes as the previous call on this
    workspace, other q / caches / out.  Reuses the set-up the workspace holds."""
    lib = load()
    total_q, Hq, D = q.shape
    total_kv, Hkv, _ = k_cache.shape
    B = q_indptr.numel() - 1
    if q_indptr.dtype != torch.int32 or kv_indptr.dtype != torch.int64:
        raise TypeError("q_indptr must be int32 and kv_indptr int64")
    if tree_mask is not None and (tree_mask.element_size() != 8 or tree_mask.numel() != total_q):
        raise TypeError("tree_mask must hold one 64-bit word per query row")
    if lse is not None and lse.dtype != torch.float32:
        raise TypeError("lse must be float32")
    if out.dtype != q.dtype or k_cache.dtype != q.dtype or v_cache.dtype != q.dtype:
        raise TypeError("q, k_cache, v_cache and out must share one dtype")
    ws_ptr = _dev_ptr(workspace, "workspace") if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.respec_verify_attention_next_layer(
        _dev_ptr(q, "q"), _dev_ptr(k_cache, "k_cache"), _dev_ptr(v_cache, "v_cache"),
        _dev_ptr(q_indptr, "q_indptr"), _dev_ptr(kv_indptr, "kv_indptr"), _dev_ptr(tree_mask, "tree_mask"),
        _dev_ptr(out, "out"), _dev_ptr(lse, "lse"), B, total_q, total_kv, max_q_per_seq, max_kv_len, Hq, Hkv, D,
        float(sm_scale), _dtype_code(q), ws_ptr, ws_bytes, _stream_ptr(stream)))


def respec_verify_attention_tree(q, k_cache, v_cache, q_indptr, kv_indptr, tree_mask, out, lse,
                                 max_q_per_seq, max_kv_len, sm_scale, workspace, stream=None):
    """As respec_verify_attention; tree_mask [total_q] int64 (or uint64) holding the 64 mask bits."""
    lib = load()
    total_q, Hq, D = q.shape
    total_kv, Hkv, _ = k_cache.shape
    B = q_indptr.numel() - 1
    if q_indptr.dtype != torch.int32 or kv_indptr.dtype != torch.int64:
        raise TypeError("q_indptr must be int32 and kv_indptr int64")
    if tree_mask.element_size() != 8 or tree_mask.numel() != total_q:
        raise TypeError("tree_mask must hold one 64-bit word per query row")
    if lse is not None and lse.dtype != torch.float32:
        raise TypeError("lse must be float32")
    if out.dtype != q.dtype or k_cache.dtype != q.dtype or v_cache.dtype != q.dtype:
        raise TypeError("q, k_cache, v_cache and out must share one dtype")
    ws_ptr = _dev_ptr(workspace, "workspace") if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.respec_verify_attention_tree(
        _dev_ptr(q, "q"), _dev_ptr(k_cache, "k_cache"), _dev_ptr(v_cache, "v_cache"),
        _dev_ptr(q_indptr, "q_indptr"), _dev_ptr(kv_indptr, "kv_indptr"), _dev_ptr(tree_mask, "tree_mask"),
        _dev_ptr(out, "out"), _dev_ptr(lse, "lse"), B, total_q, total_kv, max_q_per_seq, max_kv_len, Hq,
        Hkv, D, float(sm_scale), _dtype_code(q), ws_ptr, ws_bytes, _stream_ptr(stream)))


def respec_profile_mark_main(before: Optional[torch.cuda.Event], after: Optional[torch.cuda.Event]):
    """Have the next respec_verify_attention record the two events around its main kernel."""
    def handle(ev):
        if ev is None:
            return None
        if not ev.cuda_event:
            raise ValueError("the event must have been created (record it once first)")
        return ctypes.c_void_p(ev.cuda_event)
    load().respec_profile_mark_main(handle(before), handle(after))


def respec_rejection_sample_workspace_bytes(B, total_q, V, logits_dt) -> int:
    return int(load().respec_rejection_sample_workspace_bytes(B, total_q, V, logits_dt))


def respec_rejection_sample(target_logits, draft_logits, draft_tokens, q_indptr, u_accept, u_final,
                            out_tokens, out_num_accepted, out_flags, max_k, temperature,
                            workspace=None, stream=None):
    """target_logits [total_q,V], draft_logits [total_q-B,V]; outputs are written in place."""
    lib = load()
    total_q, V = target_logits.shape
    B = q_indptr.numel() - 1
    if q_indptr.dtype != torch.int32:
        raise TypeError("q_indptr must be int32")
    if out_tokens.dtype != torch.int32 or out_num_accepted.dtype != torch.int32:
        raise TypeError("out_tokens and out_num_accepted must be int32")
    if tuple(out_tokens.shape) != (B, max_k + 1) or out_num_accepted.numel() != B:
        raise ValueError("out_tokens must be [B, max_k+1] and out_num_accepted [B]")
    if u_final.dtype != torch.float32 or u_final.numel() != B:
        raise TypeError("u_final must be float32 [B]")
    n_draft = total_q - B
    if n_draft > 0:
        if draft_logits.dtype != target_logits.dtype or tuple(draft_logits.shape) != (n_draft, V):
            raise ValueError("draft_logits must be [total_q-B, V] in the target's dtype")
        if draft_tokens.dtype != torch.int32 or draft_tokens.numel() != n_draft:
            raise TypeError("draft_tokens must be int32 [total_q-B]")
        if u_accept.dtype != torch.float32 or u_accept.numel() != n_draft:
            raise TypeError("u_accept must be float32 [total_q-B]")
        ld_d = draft_logits.stride(0)
    else:
        draft_logits = draft_tokens = u_accept = None
        ld_d = V
    if target_logits.stride(1) != 1:
        raise ValueError("logits rows must be unit-stride")
    ws_ptr = _dev_ptr(workspace, "workspace") if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0

    def row_ptr(t, name):
        if t is None:
            return None
        if not t.is_cuda:
            raise ValueError(f"{name} must live on the GPU")
        return ctypes.c_void_p(t.data_ptr())

    _check(lib.respec_rejection_sample(
        row_ptr(target_logits, "target_logits"), row_ptr(draft_logits, "draft_logits"),
        _dev_ptr(draft_tokens, "draft_tokens"), _dev_ptr(q_indptr, "q_indptr"),
        _dev_ptr(u_accept, "u_accept"), _dev_ptr(u_final, "u_final"),
        _dev_ptr(out_tokens, "out_tokens"), _dev_ptr(out_num_accepted, "out_num_accepted"),
        _dev_ptr(out_flags, "out_flags"), B, total_q, max_k, V, target_logits.stride(0), ld_d,
        float(temperature), _dtype_code(target_logits), ws_ptr, ws_bytes, _stream_ptr(stream)))


def respec_rejection_sample_per_seq(target_logits, draft_logits, draft_tokens, q_indptr, u_accept, u_final,
                                    temperatures, out_tokens, out_num_accepted, out_flags, max_k, stream=None):
    """respec_rejection_sample with temperatures [B] float32 on the device (0 = greedy).
    draft_logits and u_accept may be None when every sequence that has drafts is greedy."""
    lib = load()
    total_q, V = target_logits.shape
    B = q_indptr.numel() - 1
    if q_indptr.dtype != torch.int32:
        raise TypeError("q_indptr must be int32")
    if out_tokens.dtype != torch.int32 or out_num_accepted.dtype != torch.int32:
        raise TypeError("out_tokens and out_num_accepted must be int32")
    if tuple(out_tokens.shape) != (B, max_k + 1) or out_num_accepted.numel() != B:
        raise ValueError("out_tokens must be [B, max_k+1] and out_num_accepted [B]")
    if u_final.dtype != torch.float32 or u_final.numel() != B:
        raise TypeError("u_final must be float32 [B]")
    if temperatures.dtype != torch.float32 or temperatures.numel() != B:
        raise TypeError("temperatures must be float32 [B]")
    n_draft = total_q - B
    ld_d = V
    if n_draft > 0:
        if draft_tokens.dtype != torch.int32 or draft_tokens.numel() != n_draft:
            raise TypeError("draft_tokens must be int32 [total_q-B]")
        if draft_logits is not None:
            if draft_logits.dtype != target_logits.dtype or tuple(draft_logits.shape) != (n_draft, V):
                raise ValueError("draft_logits must be [total_q-B, V] in the target's dtype")
            ld_d = draft_logits.stride(0)
        if u_accept is not None and (u_accept.dtype != torch.float32 or u_accept.numel() != n_draft):
            raise TypeError("u_accept must be float32 [total_q-B]")
    else:
        draft_logits = draft_tokens = u_accept = None
    if target_logits.stride(1) != 1:
        raise ValueError("logits rows must be unit-stride")

    def row_ptr(t, name):
        if t is None:
            return None
        if not t.is_cuda:
            raise ValueError(f"{name} must live on the GPU")
        return ctypes.c_void_p(t.data_ptr())

    _check(lib.respec_rejection_sample_per_seq(
        row_ptr(target_logits, "target_logits"), row_ptr(draft_logits, "draft_logits"),
        _dev_ptr(draft_tokens, "draft_tokens"), _dev_ptr(q_indptr, "q_indptr"),
        _dev_ptr(u_accept, "u_accept"), _dev_ptr(u_final, "u_final"), _dev_ptr(temperatures, "temperatures"),
        _dev_ptr(out_tokens, "out_tokens"), _dev_ptr(out_num_accepted, "out_num_accepted"),
        _dev_ptr(out_flags, "out_flags"), B, total_q, max_k, V, target_logits.stride(0), ld_d,
        _dtype_code(target_logits), _stream_ptr(stream)))


def respec_tree_rejection_sample(target_logits, draft_logits, node_tokens, parent, q_indptr, u_accept,
                                 u_final, out_tokens, out_path, out_num_accepted, out_flags,
                                 max_q_per_seq, max_depth, temperature, stream=None):
    """target_logits and draft_logits [total_q,V] (one row per tree node); outputs are written in place."""
    lib = load()
    total_q, V = target_logits.shape
    B = q_indptr.numel() - 1
    if q_indptr.dtype != torch.int32:
        raise TypeError("q_indptr must be int32")
    if draft_logits.dtype != target_logits.dtype or tuple(draft_logits.shape) != (total_q, V):
        raise ValueError("draft_logits must be [total_q, V] in the target's dtype")
    for t, name in ((node_tokens, "node_tokens"), (parent, "parent")):
        if t.dtype != torch.int32 or t.numel() != total_q:
            raise TypeError(f"{name} must be int32 [total_q]")
    if u_accept.dtype != torch.float32 or u_accept.numel() != total_q:
        raise TypeError("u_accept must be float32 [total_q]")
    if u_final.dtype != torch.float32 or u_final.numel() != B:
        raise TypeError("u_final must be float32 [B]")
    for t, name in ((out_tokens, "out_tokens"), (out_path, "out_path"), (out_num_accepted, "out_num_accepted")):
        if t.dtype != torch.int32:
            raise TypeError(f"{name} must be int32")
    if tuple(out_tokens.shape) != (B, max_depth + 1) or tuple(out_path.shape) != (B, max(max_depth, 1)):
        raise ValueError("out_tokens must be [B, max_depth+1] and out_path [B, max(max_depth,1)]")
    if out_num_accepted.numel() != B:
        raise ValueError("out_num_accepted must be [B]")
    if target_logits.stride(1) != 1 or draft_logits.stride(1) != 1:
        raise ValueError("logits rows must be unit-stride")
    for t, name in ((target_logits, "target_logits"), (draft_logits, "draft_logits")):
        if not t.is_cuda:
            raise ValueError(f"{name} must live on the GPU")
    _check(lib.respec_tree_rejection_sample(
        ctypes.c_void_p(target_logits.data_ptr()), ctypes.c_void_p(draft_logits.data_ptr()),
        _dev_ptr(node_tokens, "node_tokens"), _dev_ptr(parent, "parent"), _dev_ptr(q_indptr, "q_indptr"),
        _dev_ptr(u_accept, "u_accept"), _dev_ptr(u_final, "u_final"), _dev_ptr(out_tokens, "out_tokens"),
        _dev_ptr(out_path, "out_path"), _dev_ptr(out_num_accepted, "out_num_accepted"),
        _dev_ptr(out_flags, "out_flags"), B, total_q, max_q_per_seq, max_depth, V,
        target_logits.stride(0), draft_logits.stride(0), float(temperature), _dtype_code(target_logits),
        _stream_ptr(stream)))


def respec_verify_attention_paged_next_layer(q, k_pages, v_pages, q_indptr, page_indptr, page_table, kv_len, out,
                                             lse, max_q_per_seq, max_kv_len, sm_scale, workspace, tree_mask=None,
                                             stream=None):
    """Another layer's pools behind the same page table: reuses the set-up in the workspace."""
    respec_verify_attention_paged(q, k_pages, v_pages, q_indptr, page_indptr, page_table, kv_len, out, lse,
                                  max_q_per_seq, max_kv_len, sm_scale, workspace, tree_mask=tree_mask, stream=stream,
                                  _entry="respec_verify_attention_paged_next_layer")


def respec_verify_attention_paged(q, k_pages, v_pages, q_indptr, page_indptr, page_table, kv_len, out, lse,
                                  max_q_per_seq, max_kv_len, sm_scale, workspace, tree_mask=None, stream=None,
                                  _entry="respec_verify_attention_paged"):
    """k_pages, v_pages [num_pages, page_size, Hkv, D]; out is written in place."""
    lib = load()
    total_q, Hq, D = q.shape
    num_pages, page_size, Hkv, Dk = k_pages.shape
    if Dk != D or tuple(v_pages.shape) != tuple(k_pages.shape):
        raise ValueError("k_pages and v_pages must be [num_pages, page_size, Hkv, D] with q's D")
    if k_pages.dtype != q.dtype or v_pages.dtype != q.dtype or out.dtype != q.dtype:
        raise TypeError("q, k_pages, v_pages and out must share one dtype")
    if tuple(out.shape) != tuple(q.shape):
        raise ValueError("out must have q's shape")
    B = q_indptr.numel() - 1
    for t, name, n in ((q_indptr, "q_indptr", B + 1), (page_indptr, "page_indptr", B + 1), (kv_len, "kv_len", B)):
        if t.dtype != torch.int32 or t.numel() != n:
            raise TypeError(f"{name} must be int32 [{n}]")
    if page_table.dtype != torch.int32:
        raise TypeError("page_table must be int32")
    if tree_mask is not None and (tree_mask.dtype != torch.int64 or tree_mask.numel() != total_q):
        raise TypeError("tree_mask must be int64 [total_q] (the bits of a uint64 per row)")
    if lse is not None and (lse.dtype != torch.float32 or tuple(lse.shape) != (total_q, Hq)):
        raise TypeError("lse must be float32 [total_q, Hq]")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(getattr(lib, _entry)(
        _dev_ptr(q, "q"), _dev_ptr(k_pages, "k_pages"), _dev_ptr(v_pages, "v_pages"), _dev_ptr(q_indptr, "q_indptr"),
        _dev_ptr(page_indptr, "page_indptr"), _dev_ptr(page_table, "page_table"), _dev_ptr(kv_len, "kv_len"),
        _dev_ptr(tree_mask, "tree_mask"), _dev_ptr(out, "out"), _dev_ptr(lse, "lse"), B, total_q, num_pages,
        page_table.numel(), page_size, max_q_per_seq, max_kv_len, Hq, Hkv, D, float(sm_scale), _dtype_code(q),
        _dev_ptr(workspace, "workspace"), ws_bytes, _stream_ptr(stream)))


def respec_commit_accepted_paged(k_pages, v_pages, q_indptr, page_indptr, page_table, kv_len, num_accepted,
                                 total_q, max_q_per_seq, path=None, stream=None):
    """Moves the K/V of the accepted rows behind the last committed token; k_pages, v_pages and
    kv_len are changed in place."""
    lib = load()
    num_pages, page_size, Hkv, D = k_pages.shape
    if tuple(v_pages.shape) != tuple(k_pages.shape) or v_pages.dtype != k_pages.dtype:
        raise ValueError("k_pages and v_pages must have one shape and dtype")
    B = q_indptr.numel() - 1
    for t, name, n in ((q_indptr, "q_indptr", B + 1), (page_indptr, "page_indptr", B + 1), (kv_len, "kv_len", B),
                       (num_accepted, "num_accepted", B)):
        if t.dtype != torch.int32 or t.numel() != n:
            raise TypeError(f"{name} must be int32 [{n}]")
    if page_table.dtype != torch.int32:
        raise TypeError("page_table must be int32")
    stride = 0
    if path is not None:
        if path.dtype != torch.int32 or path.dim() != 2 or path.shape[0] != B:
            raise TypeError("path must be int32 [B, stride]")
        stride = path.shape[1]
    _check(lib.respec_commit_accepted_paged(
        _dev_ptr(k_pages, "k_pages"), _dev_ptr(v_pages, "v_pages"), _dev_ptr(q_indptr, "q_indptr"),
        _dev_ptr(page_indptr, "page_indptr"), _dev_ptr(page_table, "page_table"), _dev_ptr(kv_len, "kv_len"),
        _dev_ptr(path, "path"), stride, _dev_ptr(num_accepted, "num_accepted"), B, total_q, max_q_per_seq,
        num_pages, page_table.numel(), page_size, Hkv, D, _dtype_code(k_pages), _stream_ptr(stream)))


def respec_kd_rows_workspace_bytes(rows, V, dt) -> int:
    return int(load().respec_kd_rows_workspace_bytes(rows, V, dt))


def respec_kd_rows(target_logits, draft_logits, row_weight, grad, row_loss, total_loss, workspace, stream=None):
    """target_logits, draft_logits, grad [rows, V]; row_weight, row_loss [rows] f32; total_loss [1] f64 or None."""
    lib = load()
    rows, V = target_logits.shape
    for t, name in ((draft_logits, "draft_logits"), (grad, "grad")):
        if tuple(t.shape) != (rows, V) or t.dtype != target_logits.dtype or t.stride(1) != 1:
            raise ValueError(f"{name} must be [rows, V] in the target's dtype with unit-stride rows")
    if target_logits.stride(1) != 1:
        raise ValueError("logits rows must be unit-stride")
    for t, name in ((row_weight, "row_weight"), (row_loss, "row_loss")):
        if t.dtype != torch.float32 or t.numel() != rows:
            raise TypeError(f"{name} must be float32 [rows]")
    if total_loss is not None and (total_loss.dtype != torch.float64 or total_loss.numel() != 1):
        raise TypeError("total_loss must be float64 [1]")
    for t, name in ((target_logits, "target_logits"), (draft_logits, "draft_logits"), (grad, "grad")):
        if not t.is_cuda:
            raise ValueError(f"{name} must live on the GPU")
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.respec_kd_rows(
        ctypes.c_void_p(target_logits.data_ptr()), ctypes.c_void_p(draft_logits.data_ptr()),
        _dev_ptr(row_weight, "row_weight"), ctypes.c_void_p(grad.data_ptr()), _dev_ptr(row_loss, "row_loss"),
        _dev_ptr(total_loss, "total_loss"), rows, V, target_logits.stride(0), draft_logits.stride(0),
        grad.stride(0), _dtype_code(target_logits), _dev_ptr(workspace, "workspace"), ws_bytes,
        _stream_ptr(stream)))


def respec_solver_pick(points, active_batch, draft_us_fixed, draft_us_per_seq):
    """points: iterable of (batch, k, step_us, emitted_per_seq), host numbers.
    Returns (best_k, speedup, cost_us)."""
    lib = load()
    pts = list(points)
    arr = (ProfilePoint * max(len(pts), 1))()
    for i, (B, k, t, e) in enumerate(pts):
        arr[i] = ProfilePoint(int(B), int(k), float(t), float(e))
    best, speedup, cost = ctypes.c_int32(-1), ctypes.c_double(0.0), ctypes.c_double(0.0)
    _check(lib.respec_solver_pick(ctypes.cast(arr, ctypes.c_void_p) if pts else None, len(pts), int(active_batch),
                                  float(draft_us_fixed), float(draft_us_per_seq), ctypes.byref(best),
                                  ctypes.byref(speedup), ctypes.byref(cost)))
    return best.value, speedup.value, cost.value


def respec_validate_batch(q_indptr, kv_indptr, draft_tokens, total_q, total_kv, max_q_per_seq, max_kv_len, V,
                          stream=None):
    """Debug check of a batch's index arrays and drafted tokens; raises RespecError naming the
    first bad sequence.  Synchronises the stream."""
    lib = load()
    B = q_indptr.numel() - 1
    if q_indptr.dtype != torch.int32 or (kv_indptr is not None and kv_indptr.dtype != torch.int64):
        raise TypeError("q_indptr must be int32 and kv_indptr int64")
    if draft_tokens is not None and draft_tokens.dtype != torch.int32:
        raise TypeError("draft_tokens must be int32")
    ws = torch.empty(int(lib.respec_validate_batch_workspace_bytes(B)), dtype=torch.uint8, device=q_indptr.device)
    _check(lib.respec_validate_batch(_dev_ptr(q_indptr, "q_indptr"), _dev_ptr(kv_indptr, "kv_indptr"),
                                     _dev_ptr(draft_tokens, "draft_tokens"), B, int(total_q), int(total_kv),
                                     int(max_q_per_seq), int(max_kv_len), int(V), _dev_ptr(ws, "workspace"),
                                     ws.numel(), _stream_ptr(stream)))
