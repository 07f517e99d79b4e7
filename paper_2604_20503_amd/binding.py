"""ctypes binding of the C ABI declared in ``include/faser_verify.h``.

Argument marshalling only: tensors are checked for device, dtype and contiguity and handed
over as raw pointers together with the current HIP stream.  No arithmetic happens here and
there is no fallback: if the library is missing, the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfaser_verify.so")
_lib = None

F32, BF16 = 0, 1
PROBS, LOGITS, GREEDY = 0, 1, 2
KV_HEAD_MAJOR, KV_TOKEN_MAJOR = 0, 1
EWS = -4  # FSR_EWS: workspace missing, too small, or (binding only) still in use on another stream

SYMBOLS = [
    "fsr_last_error", "fsr_version", "fsr_attn_workspace_bytes", "fsr_attn_path", "fsr_attn_plan_bytes", "fsr_attn_plan",
    "fsr_verify_attention_planned", "fsr_verify_attention_static", "fsr_static_scratch_bytes", "fsr_verify_attention", "fsr_verify_attention_kv8", "fsr_verify_attention_kv8_planned", "fsr_kv_append", "fsr_kv_append_kv8",
    "fsr_accept_workspace_bytes", "fsr_spec_accept", "fsr_prune_compact", "fsr_prune_restore",
    "fsr_prune_scatter", "fsr_survivor_mask", "fsr_survivor_compact", "fsr_topk_rank_check", "fsr_frontier_init", "fsr_frontier_plan", "fsr_frontier_commit",
    "fsr_hbm_read_probe",
]


class FsrError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"faser_verify error {code}: {msg}")
        self.code = code


class AttnParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "N_cap", "H_q", "H_kv", "D", "P", "max_pages", "n_pages", "dtype", "out_dtype")] + \
               [("scale", ctypes.c_float), ("max_q_len", ctypes.c_int32), ("max_workgroups", ctypes.c_int32),
                ("kv_layout", ctypes.c_int32)]


class AcceptParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("V", ctypes.c_int32), ("S_max", ctypes.c_int32), ("mode", ctypes.c_int32),
                ("temperature", ctypes.c_double), ("dtype", ctypes.c_int32), ("reserved2", ctypes.c_int32)]


class PruneParams(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("N_cap", ctypes.c_int32), ("suffix_close", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


class RankParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("B", "N_cap", "D_cap", "V", "K", "dtype", "reserved")]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load ``libfaser_verify.so``; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python paper_2604_20503_amd/build.py` "
                "(there is no CPU or PyTorch fallback for the verification kernels)")
        lib = ctypes.CDLL(_LIB_PATH)
        lib.fsr_last_error.restype = ctypes.c_char_p
        lib.fsr_version.restype = ctypes.c_char_p
        for name in SYMBOLS[2:]:
            getattr(lib, name).restype = ctypes.c_int
        lib.fsr_static_scratch_bytes.restype = ctypes.c_size_t
        _lib = lib
    return _lib


def version() -> str:
    return load_library().fsr_version().decode()


def last_error() -> str:
    return load_library().fsr_last_error().decode()


def _check(rc: int):
    if rc != 0:
        raise FsrError(rc, last_error())


def _ptr(t: Optional[torch.Tensor], dtype=None, name="tensor"):
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _code(dt: torch.dtype) -> int:
    if dt == torch.float32:
        return F32
    if dt == torch.bfloat16:
        return BF16
    raise ValueError(f"unsupported dtype {dt}")


def _attn_params(q, k_cache, block_tables, B, out_dtype, scale, max_q_len, max_workgroups=0,
                 kv_layout=KV_HEAD_MAJOR) -> AttnParams:
    N_cap, H_q, D = q.shape
    if kv_layout == KV_TOKEN_MAJOR:
        n_pages, P, H_kv, D2 = k_cache.shape
    else:
        n_pages, H_kv, P, D2 = k_cache.shape
    if D2 != D:
        raise ValueError("head dim of q and k_cache differ")
    return AttnParams(B=B, N_cap=N_cap, H_q=H_q, H_kv=H_kv, D=D, P=P, max_pages=block_tables.shape[1],
                      n_pages=n_pages, dtype=_code(q.dtype), out_dtype=_code(out_dtype), scale=float(scale),
                      max_q_len=int(max_q_len), max_workgroups=int(max_workgroups), kv_layout=int(kv_layout))


def attn_workspace_bytes(*, B, N_cap, H_q, H_kv, D, P, max_pages, n_pages, dtype, out_dtype, scale=1.0,
                         max_q_len=0) -> int:
    p = AttnParams(B=B, N_cap=N_cap, H_q=H_q, H_kv=H_kv, D=D, P=P, max_pages=max_pages, n_pages=n_pages,
                   dtype=_code(dtype), out_dtype=_code(out_dtype), scale=float(scale), max_q_len=int(max_q_len),
                   max_workgroups=0, kv_layout=0)
    out = ctypes.c_size_t(0)
    _check(load_library().fsr_attn_workspace_bytes(ctypes.byref(p), ctypes.byref(out)))
    return int(out.value)


PATH_GENERIC, PATH_STREAM = 0, 1


def attn_path(*, B, N_cap, H_q, H_kv, D, P, max_pages, n_pages, dtype, out_dtype, max_q_len=0) -> int:
    """fsr_attn_path: PATH_STREAM (the bandwidth kernel) or PATH_GENERIC (one wavefront per row and head)."""
    p = AttnParams(B=B, N_cap=N_cap, H_q=H_q, H_kv=H_kv, D=D, P=P, max_pages=max_pages, n_pages=n_pages,
                   dtype=_code(dtype), out_dtype=_code(out_dtype), scale=1.0, max_q_len=int(max_q_len),
                   max_workgroups=0, kv_layout=0)
    rc = load_library().fsr_attn_path(ctypes.byref(p))
    if rc < 0:
        _check(rc)
    return rc


def attn_plan(q, k_cache, block_tables, ctx_lens, cu_q, *, scale, out_dtype=None, max_q_len=0, max_workgroups=0,
              kv_layout=KV_HEAD_MAJOR, plan=None):
    """fsr_attn_plan: build the step's schedule (device buffer, returned) for verify_attention(..., plan=...).
    q and k_cache are looked at for their shapes only."""
    lib = load_library()
    B = ctx_lens.shape[0]
    p = _attn_params(q, k_cache, block_tables, B, out_dtype or q.dtype, scale, max_q_len, max_workgroups, kv_layout)
    need = ctypes.c_size_t(0)
    _check(lib.fsr_attn_plan_bytes(ctypes.byref(p), ctypes.byref(need)))
    if plan is None:
        plan = torch.empty(max(need.value, 16), dtype=torch.uint8, device=q.device)
    _check(lib.fsr_attn_plan(_ptr(block_tables, torch.int32, "block_tables"), _ptr(ctx_lens, torch.int32, "ctx_lens"),
                             _ptr(cu_q, torch.int32, "cu_q"), ctypes.byref(p), _ptr(plan, name="plan"),
                             ctypes.c_size_t(plan.numel() * plan.element_size()), _stream()))
    return plan


# One attention call in flight per workspace (the pieces of items cut by share boundaries go through it):
# a caller-supplied workspace that was last used on another stream is refused while that stream's call
# may still be running.  Workspaces used under HIP-graph capture are not tracked (no event can be recorded).
_ws_last_use = {}


def _guard_workspace(workspace):
    if workspace is None or torch.cuda.is_current_stream_capturing():
        return None
    key = workspace.data_ptr()
    stream = torch.cuda.current_stream()
    last = _ws_last_use.get(key)
    if last is not None and last[0] != stream.cuda_stream and not last[1].query():
        raise FsrError(EWS, "this attention workspace is still in use by a call on another stream: "
                                     "give every stream (and every graph that may replay concurrently) its own workspace")
    return key, stream


def _note_workspace_use(token):
    if token is not None:
        key, stream = token
        ev = torch.cuda.Event()
        ev.record(stream)
        _ws_last_use[key] = (stream.cuda_stream, ev)


def verify_attention(q, k_cache, v_cache, block_tables, ctx_lens, spec_lens, cu_q, *, scale, out=None, lse=None,
                     out_dtype=None, workspace=None, max_q_len=0, max_workgroups=0, kv_layout=KV_HEAD_MAJOR, plan=None):
    """fsr_verify_attention.  q [N_cap,H_q,D]; caches [n_pages,H_kv,P,D]; returns (out, lse).
    max_workgroups: size of the persistent grid when the current stream owns only part of the device.
    kv_layout: KV_HEAD_MAJOR (caches [n_pages,H_kv,P,D]) or KV_TOKEN_MAJOR (caches [n_pages,P,H_kv,D]).
    plan: buffer from attn_plan for the same shapes and metadata -> fsr_verify_attention_planned."""
    lib = load_library()
    B = ctx_lens.shape[0]
    out_dtype = out_dtype or (out.dtype if out is not None else q.dtype)
    p = _attn_params(q, k_cache, block_tables, B, out_dtype, scale, max_q_len, max_workgroups, kv_layout)
    if out is None:
        out = torch.empty(q.shape, dtype=out_dtype, device=q.device)
    if v_cache.shape != k_cache.shape or v_cache.dtype != k_cache.dtype or k_cache.dtype != q.dtype:
        raise ValueError("q, k_cache and v_cache must share dtype; caches must share shape")
    if cu_q.shape[0] != B + 1 or block_tables.shape[0] != B:
        raise ValueError("cu_q must have B+1 entries and block_tables B rows")
    need = ctypes.c_size_t(0)
    _check(lib.fsr_attn_workspace_bytes(ctypes.byref(p), ctypes.byref(need)))
    token = _guard_workspace(workspace)
    if workspace is None and need.value:
        workspace = torch.empty(need.value, dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if plan is not None:
        _check(lib.fsr_verify_attention_planned(
            _ptr(q, name="q"), _ptr(k_cache, name="k_cache"), _ptr(v_cache, name="v_cache"),
            _ptr(block_tables, torch.int32, "block_tables"), _ptr(ctx_lens, torch.int32, "ctx_lens"),
            _ptr(cu_q, torch.int32, "cu_q"), _ptr(out, name="out"), _ptr(lse, torch.float32, "lse"), ctypes.byref(p),
            _ptr(plan, name="plan"), _ptr(workspace, name="workspace"), ctypes.c_size_t(ws_bytes), _stream()))
        _note_workspace_use(token)
        return out, lse
    _check(lib.fsr_verify_attention(
        _ptr(q, name="q"), _ptr(k_cache, name="k_cache"), _ptr(v_cache, name="v_cache"),
        _ptr(block_tables, torch.int32, "block_tables"), _ptr(ctx_lens, torch.int32, "ctx_lens"),
        _ptr(spec_lens, torch.int32, "spec_lens"), _ptr(cu_q, torch.int32, "cu_q"), _ptr(out, name="out"),
        _ptr(lse, torch.float32, "lse"), ctypes.byref(p), _ptr(workspace, name="workspace"),
        ctypes.c_size_t(ws_bytes), _stream()))
    _note_workspace_use(token)
    return out, lse


def verify_attention_static(q, k_cache, v_cache, block_tables, ctx_lens, cu_q, *, scale, out, lse=None, max_q_len=0,
                            max_workgroups=0, kv_layout=KV_HEAD_MAJOR):
    """fsr_verify_attention_static: no workspace argument and no allocation, here or in the library (`out` is
    the caller's).  Returns (out, lse)."""
    B = ctx_lens.shape[0]
    p = _attn_params(q, k_cache, block_tables, B, out.dtype, scale, max_q_len, max_workgroups, kv_layout)
    if v_cache.shape != k_cache.shape or v_cache.dtype != k_cache.dtype or k_cache.dtype != q.dtype:
        raise ValueError("q, k_cache and v_cache must share dtype; caches must share shape")
    if cu_q.shape[0] != B + 1 or block_tables.shape[0] != B or out.shape != q.shape:
        raise ValueError("cu_q must have B+1 entries, block_tables B rows, out the shape of q")
    _check(load_library().fsr_verify_attention_static(
        _ptr(q, name="q"), _ptr(k_cache, name="k_cache"), _ptr(v_cache, name="v_cache"),
        _ptr(block_tables, torch.int32, "block_tables"), _ptr(ctx_lens, torch.int32, "ctx_lens"),
        _ptr(cu_q, torch.int32, "cu_q"), _ptr(out, name="out"), _ptr(lse, torch.float32, "lse"), ctypes.byref(p), _stream()))
    return out, lse


def verify_attention_kv8(q, k_cache, v_cache, k_scale, v_scale, block_tables, ctx_lens, cu_q, *, scale, out=None, lse=None,
                         out_dtype=None, workspace=None, max_q_len=0, max_workgroups=0, kv_layout=KV_HEAD_MAJOR, plan=None):
    """fsr_verify_attention_kv8: caches are uint8 tensors of E4M3 bytes, k_scale / v_scale [H_kv] float32.
    plan: buffer from attn_plan for the same shapes and metadata -> fsr_verify_attention_kv8_planned."""
    lib = load_library()
    B = ctx_lens.shape[0]
    out_dtype = out_dtype or (out.dtype if out is not None else q.dtype)
    p = _attn_params(q, k_cache, block_tables, B, out_dtype, scale, max_q_len, max_workgroups, kv_layout)
    if out is None:
        out = torch.empty(q.shape, dtype=out_dtype, device=q.device)
    if v_cache.shape != k_cache.shape or k_cache.dtype != torch.uint8 or v_cache.dtype != torch.uint8:
        raise ValueError("caches must be uint8 tensors of one shape")
    if k_scale.shape[0] != p.H_kv or v_scale.shape[0] != p.H_kv:
        raise ValueError("k_scale and v_scale need one entry per KV head")
    if cu_q.shape[0] != B + 1 or block_tables.shape[0] != B:
        raise ValueError("cu_q must have B+1 entries and block_tables B rows")
    need = ctypes.c_size_t(0)
    _check(lib.fsr_attn_workspace_bytes(ctypes.byref(p), ctypes.byref(need)))
    if workspace is None and need.value:
        workspace = torch.empty(need.value, dtype=torch.uint8, device=q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if plan is not None:
        _check(lib.fsr_verify_attention_kv8_planned(
            _ptr(q, name="q"), _ptr(k_cache, name="k_cache"), _ptr(v_cache, name="v_cache"),
            _ptr(k_scale, torch.float32, "k_scale"), _ptr(v_scale, torch.float32, "v_scale"),
            _ptr(block_tables, torch.int32, "block_tables"), _ptr(ctx_lens, torch.int32, "ctx_lens"),
            _ptr(cu_q, torch.int32, "cu_q"), _ptr(out, name="out"), _ptr(lse, torch.float32, "lse"), ctypes.byref(p),
            _ptr(plan, name="plan"), _ptr(workspace, name="workspace"), ctypes.c_size_t(ws_bytes), _stream()))
        return out, lse
    _check(lib.fsr_verify_attention_kv8(
        _ptr(q, name="q"), _ptr(k_cache, name="k_cache"), _ptr(v_cache, name="v_cache"),
        _ptr(k_scale, torch.float32, "k_scale"), _ptr(v_scale, torch.float32, "v_scale"),
        _ptr(block_tables, torch.int32, "block_tables"), _ptr(ctx_lens, torch.int32, "ctx_lens"),
        _ptr(cu_q, torch.int32, "cu_q"), _ptr(out, name="out"), _ptr(lse, torch.float32, "lse"), ctypes.byref(p),
        _ptr(workspace, name="workspace"), ctypes.c_size_t(ws_bytes), _stream()))
    return out, lse


def kv_append(k_new, v_new, k_cache, v_cache, block_tables, ctx_lens, cu_q, *, kv_layout=KV_HEAD_MAJOR):
    """fsr_kv_append: store the call's key / value rows [N_cap, H_kv, D] into the paged caches (in place)."""
    lib = load_library()
    B = ctx_lens.shape[0]
    if kv_layout == KV_TOKEN_MAJOR:
        n_pages, P, H_kv, D = k_cache.shape
    else:
        n_pages, H_kv, P, D = k_cache.shape
    if k_new.shape != v_new.shape or k_new.shape[1:] != (H_kv, D) or v_cache.shape != k_cache.shape:
        raise ValueError("k_new/v_new must be [N_cap, H_kv, D] matching the caches")
    if not (k_new.dtype == v_new.dtype == k_cache.dtype == v_cache.dtype):
        raise ValueError("k_new, v_new and the caches must share a dtype")
    p = AttnParams(B=B, N_cap=k_new.shape[0], H_q=H_kv, H_kv=H_kv, D=D, P=P, max_pages=block_tables.shape[1],
                   n_pages=n_pages, dtype=_code(k_new.dtype), out_dtype=_code(k_new.dtype), scale=1.0, max_q_len=0,
                   max_workgroups=0, kv_layout=int(kv_layout))
    _check(lib.fsr_kv_append(_ptr(k_new, name="k_new"), _ptr(v_new, name="v_new"), _ptr(k_cache, name="k_cache"),
                             _ptr(v_cache, name="v_cache"), _ptr(block_tables, torch.int32, "block_tables"),
                             _ptr(ctx_lens, torch.int32, "ctx_lens"), _ptr(cu_q, torch.int32, "cu_q"), ctypes.byref(p),
                             _stream()))


def kv_append_kv8(k_new, v_new, k_cache, v_cache, k_scale, v_scale, block_tables, ctx_lens, cu_q, *, kv_layout=KV_HEAD_MAJOR):
    """fsr_kv_append_kv8: quantise the call's bf16 key / value rows to E4M3 and store them into the uint8 caches."""
    lib = load_library()
    B = ctx_lens.shape[0]
    p = _attn_params(k_new, k_cache, block_tables, B, k_new.dtype, 1.0, 0, 0, kv_layout)
    if v_new.shape != k_new.shape or v_cache.shape != k_cache.shape or k_cache.dtype != torch.uint8 or v_cache.dtype != torch.uint8:
        raise ValueError("rows must share a shape; caches must be uint8 tensors of one shape")
    _check(lib.fsr_kv_append_kv8(
        _ptr(k_new, name="k_new"), _ptr(v_new, name="v_new"), _ptr(k_cache, name="k_cache"), _ptr(v_cache, name="v_cache"),
        _ptr(k_scale, torch.float32, "k_scale"), _ptr(v_scale, torch.float32, "v_scale"),
        _ptr(block_tables, torch.int32, "block_tables"), _ptr(ctx_lens, torch.int32, "ctx_lens"),
        _ptr(cu_q, torch.int32, "cu_q"), ctypes.byref(p), _stream()))


def accept_workspace_bytes(*, B, V, S_max, mode=PROBS, temperature=1.0) -> int:
    p = AcceptParams(B=B, V=V, S_max=S_max, mode=mode, temperature=float(temperature), dtype=F32, reserved2=0)
    out = ctypes.c_size_t(0)
    _check(load_library().fsr_accept_workspace_bytes(ctypes.byref(p), ctypes.byref(out)))
    return int(out.value)


def spec_accept(p_target, p_draft, draft_tokens, u_accept, u_sample, cu_t, cu_d, *, S_max, t_rows=None, d_rows=None,
                mode=PROBS, temperature=1.0, accepted_len=None, n_emitted=None, emitted=None, workspace=None):
    """fsr_spec_accept.  Returns (accepted_len [B], n_emitted [B], emitted [B, S_max+1])."""
    lib = load_library()
    B = cu_t.shape[0] - 1
    V = p_target.shape[1]
    dev = p_target.device
    if p_draft is not None and p_draft.dtype != p_target.dtype:
        raise ValueError("p_target and p_draft must share a dtype")
    p = AcceptParams(B=B, V=V, S_max=S_max, mode=mode, temperature=float(temperature), dtype=_code(p_target.dtype),
                     reserved2=0)
    if accepted_len is None:
        accepted_len = torch.empty(B, dtype=torch.int32, device=dev)
    if n_emitted is None:
        n_emitted = torch.empty(B, dtype=torch.int32, device=dev)
    if emitted is None:
        emitted = torch.empty((B, S_max + 1), dtype=torch.int32, device=dev)
    if emitted.shape != (B, S_max + 1):
        raise ValueError("emitted must be [B, S_max+1]")
    if cu_t.shape[0] != B + 1 or cu_d.shape[0] != B + 1:
        raise ValueError("cu_t and cu_d must have B+1 entries")
    need = ctypes.c_size_t(0)
    _check(lib.fsr_accept_workspace_bytes(ctypes.byref(p), ctypes.byref(need)))
    if workspace is None:
        workspace = torch.empty(max(need.value, 256), dtype=torch.uint8, device=dev)
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(lib.fsr_spec_accept(
        _ptr(p_target, name="p_target"), _ptr(p_draft, name="p_draft"),
        _ptr(draft_tokens, torch.int32, "draft_tokens"), _ptr(u_accept, torch.float32, "u_accept"),
        _ptr(u_sample, torch.float32, "u_sample"), _ptr(cu_t, torch.int32, "cu_t"), _ptr(cu_d, torch.int32, "cu_d"),
        _ptr(t_rows, torch.int32, "t_rows"), _ptr(d_rows, torch.int32, "d_rows"),
        _ptr(accepted_len, torch.int32, "accepted_len"), _ptr(n_emitted, torch.int32, "n_emitted"),
        _ptr(emitted, torch.int32, "emitted"), ctypes.byref(p), _ptr(workspace, name="workspace"),
        ctypes.c_size_t(ws_bytes), _stream()))
    return accepted_len, n_emitted, emitted


def survivor_compact(accepted_len, cu_q, N_cap, *, keep_mask=None, payload=None, payload_out=None, out=None):
    """fsr_survivor_compact: rows 0..accepted_len[i] of every request survive and are re-packed (keep_mask, if
    given, receives the mask).  Returns the dict of prune_compact."""
    return prune_compact(keep_mask, cu_q, suffix_close=True, payload=payload, payload_out=payload_out, out=out,
                         accepted_len=accepted_len, N_cap=N_cap)


def prune_compact(keep_mask, cu_q, *, suffix_close=True, payload=None, payload_out=None, out=None, accepted_len=None,
                  N_cap=None):
    """fsr_prune_compact.  Returns dict(new_cu_q, new_q_lens, src_row, dst_row, n_active, active_ids[, payload]).
    With accepted_len (and N_cap) it is fsr_survivor_compact and keep_mask an optional output."""
    lib = load_library()
    B = cu_q.shape[0] - 1
    if N_cap is None:
        N_cap = keep_mask.shape[0]
    dev = cu_q.device
    p = PruneParams(B=B, N_cap=N_cap, suffix_close=1 if suffix_close else 0, reserved=0)
    o = out or {}
    i32 = dict(dtype=torch.int32, device=dev)
    new_cu_q = o.get("new_cu_q", None)
    if new_cu_q is None:
        new_cu_q = torch.empty(B + 1, **i32)
    new_q_lens = o.get("new_q_lens") if "new_q_lens" in o else torch.empty(B, **i32)
    src_row = o.get("src_row") if "src_row" in o else torch.empty(N_cap, **i32)
    dst_row = o.get("dst_row") if "dst_row" in o else torch.empty(N_cap, **i32)
    n_active = o.get("n_active") if "n_active" in o else torch.empty(1, **i32)
    active_ids = o.get("active_ids") if "active_ids" in o else torch.empty(B, **i32)
    row_bytes = 0
    if payload is not None:
        if payload.shape[0] != N_cap:
            raise ValueError("payload must have N_cap rows")
        row_bytes = (payload.numel() // max(N_cap, 1)) * payload.element_size() if N_cap else 0
        if payload_out is None:
            payload_out = torch.empty_like(payload)
    if accepted_len is not None:
        _check(lib.fsr_survivor_compact(
            _ptr(accepted_len, torch.int32, "accepted_len"), _ptr(cu_q, torch.int32, "cu_q"),
            _ptr(keep_mask, torch.uint8, "keep_mask"), _ptr(new_cu_q, torch.int32),
            _ptr(new_q_lens, torch.int32), _ptr(src_row, torch.int32), _ptr(dst_row, torch.int32),
            _ptr(n_active, torch.int32), _ptr(active_ids, torch.int32),
            _ptr(payload if row_bytes else None, name="payload"), _ptr(payload_out if row_bytes else None, name="payload_out"),
            ctypes.c_size_t(row_bytes), ctypes.byref(p), _stream()))
        res = dict(new_cu_q=new_cu_q, new_q_lens=new_q_lens, src_row=src_row, dst_row=dst_row, n_active=n_active,
                   active_ids=active_ids)
        if payload is not None:
            res["payload"] = payload_out
        return res
    _check(lib.fsr_prune_compact(
        _ptr(keep_mask, torch.uint8, "keep_mask"), _ptr(cu_q, torch.int32, "cu_q"), _ptr(new_cu_q, torch.int32),
        _ptr(new_q_lens, torch.int32), _ptr(src_row, torch.int32), _ptr(dst_row, torch.int32),
        _ptr(n_active, torch.int32), _ptr(active_ids, torch.int32),
        _ptr(payload if row_bytes else None, name="payload"), _ptr(payload_out if row_bytes else None, name="payload_out"),
        ctypes.c_size_t(row_bytes), ctypes.byref(p), _stream()))
    res = dict(new_cu_q=new_cu_q, new_q_lens=new_q_lens, src_row=src_row, dst_row=dst_row, n_active=n_active,
               active_ids=active_ids)
    if payload is not None:
        res["payload"] = payload_out
    return res


def topk_rank_check(logits, draft_tokens, cu_q, cu_d, *, K, rank=None, keep_mask=None):
    """fsr_topk_rank_check.  logits [N_cap, V] fp32 or bf16; returns (rank [D_cap] int32, keep_mask [N_cap] uint8)."""
    lib = load_library()
    N_cap, V = logits.shape
    D_cap = draft_tokens.shape[0]
    B = cu_q.shape[0] - 1
    if cu_d.shape[0] != B + 1:
        raise ValueError("cu_q and cu_d must both have B+1 entries")
    if rank is None:
        rank = torch.empty(D_cap, dtype=torch.int32, device=logits.device)
    if keep_mask is None:
        keep_mask = torch.empty(N_cap, dtype=torch.uint8, device=logits.device)
    p = RankParams(B=B, N_cap=N_cap, D_cap=D_cap, V=V, K=int(K), dtype=_code(logits.dtype), reserved=0)
    _check(lib.fsr_topk_rank_check(
        _ptr(logits, name="logits"), _ptr(draft_tokens if D_cap else None, torch.int32, "draft_tokens"),
        _ptr(cu_q, torch.int32, "cu_q"), _ptr(cu_d, torch.int32, "cu_d"), _ptr(rank if D_cap else None, torch.int32, "rank"),
        _ptr(keep_mask, torch.uint8, "keep_mask"), ctypes.byref(p), _stream()))
    return rank, keep_mask


def prune_restore(compact, dst_row, *, pad_word=0, restored=None, has_value=None):
    """fsr_prune_restore.  Returns (restored [N, ...], has_value [N] uint8)."""
    lib = load_library()
    N = dst_row.shape[0]
    row_shape = tuple(compact.shape[1:])
    if restored is None:
        restored = torch.empty((N,) + row_shape, dtype=compact.dtype, device=compact.device)
    if has_value is None:
        has_value = torch.empty(N, dtype=torch.uint8, device=compact.device)
    row_elems = 1
    for s in row_shape:
        row_elems *= s
    row_bytes = row_elems * compact.element_size()
    _check(lib.fsr_prune_restore(_ptr(compact, name="compact"), _ptr(dst_row, torch.int32, "dst_row"),
                                 _ptr(restored, name="restored"), _ptr(has_value, torch.uint8, "has_value"),
                                 ctypes.c_size_t(row_bytes), ctypes.c_int32(N), ctypes.c_uint32(pad_word), _stream()))
    return restored, has_value


def prune_scatter(compact, src_row, n_rows, out):
    """fsr_prune_scatter: out[src_row[r]] = compact[r] for r < n_rows[0]."""
    N_cap = src_row.shape[0]
    if compact.shape[0] != N_cap or out.shape != compact.shape or out.dtype != compact.dtype:
        raise ValueError("compact and out must be [N_cap, ...] of the same shape and dtype")
    row_bytes = (compact.numel() // max(N_cap, 1)) * compact.element_size()
    _check(load_library().fsr_prune_scatter(_ptr(compact, name="compact"), _ptr(src_row, torch.int32, "src_row"),
                                            _ptr(n_rows, torch.int32, "n_rows"), _ptr(out, name="out"),
                                            ctypes.c_size_t(row_bytes), ctypes.c_int32(N_cap), _stream()))
    return out


def survivor_mask(accepted_len, cu_q, keep_mask):
    """fsr_survivor_mask: keep rows 0..accepted_len[i] of every request."""
    B = accepted_len.shape[0]
    _check(load_library().fsr_survivor_mask(_ptr(accepted_len, torch.int32, "accepted_len"), _ptr(cu_q, torch.int32, "cu_q"),
                                            _ptr(keep_mask, torch.uint8, "keep_mask"), ctypes.c_int32(B),
                                            ctypes.c_int32(keep_mask.shape[0]), _stream()))
    return keep_mask


def frontier_init(spec_lens, pos, active, n_out, acc_total, out_tokens):
    B = spec_lens.shape[0]
    _check(load_library().fsr_frontier_init(
        _ptr(spec_lens, torch.int32), _ptr(pos, torch.int32), _ptr(active, torch.int32), _ptr(n_out, torch.int32),
        _ptr(acc_total, torch.int32), _ptr(out_tokens, torch.int32), ctypes.c_int32(B),
        ctypes.c_int32(out_tokens.shape[1]), _stream()))


def frontier_plan(ctx_lens, spec_lens, cu_q, cu_d, pos, active, chunk_len, t_mask, d_mask, chunk_ctx):
    B = spec_lens.shape[0]
    _check(load_library().fsr_frontier_plan(
        _ptr(ctx_lens, torch.int32), _ptr(spec_lens, torch.int32), _ptr(cu_q, torch.int32), _ptr(cu_d, torch.int32),
        _ptr(pos, torch.int32), _ptr(active, torch.int32), _ptr(chunk_len, torch.int32), _ptr(t_mask, torch.uint8),
        _ptr(d_mask, torch.uint8), _ptr(chunk_ctx, torch.int32), ctypes.c_int32(B), ctypes.c_int32(t_mask.shape[0]),
        ctypes.c_int32(d_mask.shape[0]), _stream()))


def frontier_commit(spec_lens, chunk_len, accepted_len, n_emitted, emitted, pos, active, n_out, acc_total, out_tokens):
    B = spec_lens.shape[0]
    _check(load_library().fsr_frontier_commit(
        _ptr(spec_lens, torch.int32), _ptr(chunk_len, torch.int32), _ptr(accepted_len, torch.int32),
        _ptr(n_emitted, torch.int32), _ptr(emitted, torch.int32), ctypes.c_int32(emitted.shape[1]),
        _ptr(pos, torch.int32), _ptr(active, torch.int32), _ptr(n_out, torch.int32), _ptr(acc_total, torch.int32),
        _ptr(out_tokens, torch.int32), ctypes.c_int32(B), ctypes.c_int32(out_tokens.shape[1]), _stream()))


def hbm_read_probe(src: torch.Tensor, sink: Optional[torch.Tensor] = None, workgroups: int = 4096, scatter_4k: int = 0):
    """fsr_hbm_read_probe: one launch that streams all of ``src`` (device bytes, a multiple of 32768) with
    plain loads: front to back (0), in scattered 4 KB blocks (1), or those blocks as 64-byte segments of 16
    rows per load (2); returns the sink tensor (int64 [workgroups]).  Measurement aid for bench.py."""
    lib = load_library()
    if sink is None:
        sink = torch.empty(workgroups, dtype=torch.int64, device=src.device)
    _check(lib.fsr_hbm_read_probe(_ptr(src, name="src"), ctypes.c_size_t(src.numel() * src.element_size()),
                                  _ptr(sink, torch.int64, name="sink"), ctypes.c_int32(workgroups), ctypes.c_int32(int(scatter_4k)), _stream()))
    return sink
