"""Thin ctypes binding of libobcache.so (C ABI in include/obcache.h).

Argument marshalling only: tensors in, device pointers and sizes out.  Every step of
the path runs in the HIP kernels; torch supplies device memory and the current
stream.  There is no CPU fallback: a missing library is built once with hipcc, and a
failure to build or load it raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libobcache.so")

OBC_VALUE, OBC_KEY, OBC_JOINT, OBC_ALL, OBC_ATTN, OBC_VATP = 0, 1, 2, 3, 4, 5
OBC_F32, OBC_BF16 = 0, 1
OBC_OK, OBC_EINVAL, OBC_EUNSUPPORTED, OBC_EWORKSPACE, OBC_ELAUNCH = 0, -1, -2, -3, -4
VARIANT_CODES = {"value": OBC_VALUE, "key": OBC_KEY, "joint": OBC_JOINT, "all": OBC_ALL, "attn": OBC_ATTN,
                 "vatp": OBC_VATP}

_lib = None


class ObcError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s" % (where, obc_status_string(status)))


def load_library():
    """Loads (building first if absent) the HIP library and declares the ABI signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build_library()
    lib = ctypes.CDLL(LIB_PATH)
    c_int, c_void_p, c_size_t = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.obc_version.restype = c_int
    lib.obc_status_string.restype = ctypes.c_char_p
    lib.obc_status_string.argtypes = [c_int]
    lib.obc_score_workspace_bytes.restype = c_int
    lib.obc_score_workspace_bytes.argtypes = [c_int] * 8 + [ctypes.POINTER(c_size_t)]
    lib.obc_score.restype = c_int
    lib.obc_score.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_void_p,
                              c_int, c_int, i32p, c_void_p, c_size_t, c_void_p]
    lib.obc_score_accumulate.restype = c_int
    lib.obc_score_accumulate.argtypes = lib.obc_score.argtypes
    lib.obc_score_stages.restype = c_int
    lib.obc_score_stages.argtypes = lib.obc_score.argtypes + [c_int]
    lib.obc_select.restype = c_int
    lib.obc_select.argtypes = [c_void_p, c_int, c_void_p, c_int, c_int, c_int, i32p, c_void_p, c_size_t, c_void_p]
    lib.obc_select_workspace_bytes.restype = c_int
    lib.obc_select_workspace_bytes.argtypes = [c_int, c_int, c_int, ctypes.POINTER(c_size_t)]
    lib.obc_select_protected.restype = c_int
    lib.obc_select_protected.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_int, c_int, c_int, i32p,
                                         c_void_p, c_size_t, c_void_p]
    lib.obc_select_pooled.restype = c_int
    lib.obc_select_pooled.argtypes = [c_void_p, c_int, c_int, c_int, c_int, c_int, c_void_p, c_int, c_int, c_int, i32p,
                                      c_void_p, c_size_t, c_void_p]
    lib.obc_select_adaptive_workspace_bytes.restype = c_int
    lib.obc_select_adaptive_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int, c_int, ctypes.POINTER(c_size_t)]
    lib.obc_select_adaptive.restype = c_int
    lib.obc_select_adaptive.argtypes = [c_void_p, c_int, c_int, c_void_p, c_void_p, c_int, c_int, c_int, c_int, i32p,
                                        c_void_p, c_size_t, c_void_p]
    lib.obc_compact.restype = c_int
    lib.obc_compact.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int,
                                c_int, c_void_p]
    lib.obc_compact_inplace.restype = c_int
    lib.obc_compact_inplace.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int,
                                        c_void_p]
    lib.obc_compact_scores.restype = c_int
    lib.obc_compact_scores.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_void_p]
    lib.obc_probe_read_bandwidth.restype = c_int
    lib.obc_probe_read_bandwidth.argtypes = [c_void_p, c_size_t, c_void_p, c_void_p]
    lib.obc_init.restype = c_int
    lib.obc_score_static.restype = c_int
    lib.obc_score_static.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_void_p,
                                     c_int, c_int, i32p, c_int, c_void_p]
    lib.obc_decode_step_workspace_bytes.restype = c_int
    lib.obc_decode_step_workspace_bytes.argtypes = [c_int] * 7 + [ctypes.POINTER(c_size_t)]
    lib.obc_decode_step.restype = c_int
    lib.obc_decode_step.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int,
                                    c_int, c_int, i32p, c_int, c_int, c_void_p, c_size_t, c_void_p]
    lib.obc_set_score_path.restype = c_int
    lib.obc_set_score_path.argtypes = [c_int]
    lib.obc_set_score_tuning.restype = c_int
    lib.obc_set_score_tuning.argtypes = [c_int, c_int]
    lib.obc_set_sweep2_form.restype = c_int
    lib.obc_set_sweep2_form.argtypes = [c_int]
    _lib = lib
    return lib


def obc_version() -> int:
    return int(load_library().obc_version())


def obc_status_string(status: int) -> str:
    return load_library().obc_status_string(int(status)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return OBC_F32
    if t.dtype == torch.bfloat16:
        return OBC_BF16
    raise TypeError("q, k, v must be float32 or bfloat16, got %s" % t.dtype)


def _lens_arg(seq_lens: Optional[Sequence[int]], B: int):
    if seq_lens is None:
        return None
    if len(seq_lens) != B:
        raise ValueError("seq_lens needs one entry per sequence")
    return (ctypes.c_int32 * B)(*[int(x) for x in seq_lens])


def _stream_ptr(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def _require_cuda(*tensors):
    for t in tensors:
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("tensors must be contiguous and on the GPU")


def obc_score_workspace_bytes(B, N, W, Hq, Hkv, d, dtype, variant) -> int:
    out = ctypes.c_size_t(0)
    rc = load_library().obc_score_workspace_bytes(B, N, W, Hq, Hkv, d, dtype, variant, ctypes.byref(out))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_score_workspace_bytes")
    return int(out.value)


OBC_STAGE_SWEEP1, OBC_STAGE_COMBINE, OBC_STAGE_SWEEP2, OBC_STAGE_ALL = 1, 2, 4, 7
PATH_CODES = {"auto": 0, "plain": 1, "mfma": 2, "decode": 3}


def obc_set_score_path(path="auto") -> None:
    """Test hook: pins the scoring kernels process-wide ("auto" | "plain" | "mfma" | "decode")."""
    rc = load_library().obc_set_score_path(PATH_CODES[path] if isinstance(path, str) else int(path))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_set_score_path")


def obc_set_sweep2_form(form: int = 0) -> None:
    """Test hook: 0 = second sweep chosen by shape, 1 = 32 rows per wave, 2 = 64 rows per wave where possible."""
    rc = load_library().obc_set_sweep2_form(int(form))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_set_sweep2_form")


def obc_set_score_tuning(splits: int = 0, range_len: int = 0) -> None:
    """Tuning hook: sweep-1 split count and sweep-2 token range of the matrix-core path (0 = automatic)."""
    rc = load_library().obc_set_score_tuning(int(splits), int(range_len))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_set_score_tuning")


def obc_score(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, variant="joint", seq_lens=None,
              scores: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
              stage_mask: Optional[int] = None, accumulate: bool = False) -> torch.Tensor:
    """q [B,Hq,W,d], k,v [B,Hkv,N,d] -> scores [B,Hkv,N] fp32 ([3,B,Hkv,N] for variant "all").

    stage_mask (measurement hook) routes the call through obc_score_stages; accumulate=True through
    obc_score_accumulate (adds to the `scores` passed in, which is then required)."""
    _require_cuda(q, k, v)
    B, Hq, W, d = q.shape
    Bk, Hkv, N, dk = k.shape
    if (Bk, dk) != (B, d) or v.shape != k.shape or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v shapes or dtypes disagree")
    var = VARIANT_CODES[variant] if isinstance(variant, str) else int(variant)
    dt = _dtype_code(q)
    if workspace is None:
        workspace = torch.empty(obc_score_workspace_bytes(B, N, W, Hq, Hkv, d, dt, var), dtype=torch.uint8,
                                device=q.device)
    shape = (3, B, Hkv, N) if var == OBC_ALL else (B, Hkv, N)
    if scores is None:
        if accumulate:
            raise ValueError("accumulate=True needs the running scores tensor")
        scores = torch.empty(shape, dtype=torch.float32, device=q.device)
    elif tuple(scores.shape) != shape or scores.dtype != torch.float32 or not scores.is_contiguous():
        raise ValueError("scores must be a contiguous float32 tensor of shape %s" % (shape,))
    _require_cuda(scores, workspace)
    args = (q.data_ptr(), k.data_ptr(), v.data_ptr(), N, W, Hq, Hkv, d, var, scores.data_ptr(), B, dt,
            _lens_arg(seq_lens, B), workspace.data_ptr(), workspace.numel(), _stream_ptr(q))
    if accumulate:
        if stage_mask is not None:
            raise ValueError("stage_mask and accumulate exclude each other")
        rc = load_library().obc_score_accumulate(*args)
    elif stage_mask is None:
        rc = load_library().obc_score(*args)
    else:
        rc = load_library().obc_score_stages(*args, int(stage_mask))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_score")
    return scores


OBC_STATIC_SCRATCH_BYTES = 48 << 20


def obc_init() -> None:
    rc = load_library().obc_init()
    if rc != OBC_OK:
        raise ObcError(rc, "obc_init")


def obc_score_static(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, variant, scores: torch.Tensor, seq_lens=None,
                     accumulate: bool = False) -> torch.Tensor:
    """obc_score / obc_score_accumulate on the library's static scratch: the caller passes inputs and the output
    tensor, and nothing is allocated (not by torch either)."""
    _require_cuda(q, k, v, scores)
    B, Hq, W, d = q.shape
    _, Hkv, N, _ = k.shape
    var = VARIANT_CODES[variant] if isinstance(variant, str) else int(variant)
    shape = (3, B, Hkv, N) if var == OBC_ALL else (B, Hkv, N)
    if tuple(scores.shape) != shape or scores.dtype != torch.float32 or v.shape != k.shape:
        raise ValueError("scores must be a contiguous float32 tensor of shape %s" % (shape,))
    rc = load_library().obc_score_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), N, W, Hq, Hkv, d, var,
                                         scores.data_ptr(), B, _dtype_code(q), _lens_arg(seq_lens, B),
                                         1 if accumulate else 0, _stream_ptr(q))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_score_static")
    return scores


def obc_select_workspace_bytes(B: int, Hkv: int, N: int) -> int:
    out = ctypes.c_size_t(0)
    rc = load_library().obc_select_workspace_bytes(B, Hkv, N, ctypes.byref(out))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_select_workspace_bytes")
    return int(out.value)


def _select_ws(scores: torch.Tensor, workspace):
    """(pointer, bytes, tensor) of the optional selection scratch; allocates it when the shape profits and none was
    given.  The caller keeps the tensor alive until its C call has enqueued the kernels: torch's allocator hands a
    freed block to the next allocation on the same stream, which is only safe after the launches that use it.
    workspace=False asks for the one-block-per-head path."""
    if workspace is False:
        return None, 0, None
    B, Hkv, N = scores.shape
    if workspace is None:
        need = obc_select_workspace_bytes(B, Hkv, N)
        if need == 0:
            return None, 0, None
        workspace = torch.empty(need, dtype=torch.uint8, device=scores.device)
    _require_cuda(workspace)
    return workspace.data_ptr(), workspace.numel(), workspace


def obc_select(scores: torch.Tensor, budget: int, seq_lens=None,
               keep_idx: Optional[torch.Tensor] = None, workspace=None) -> torch.Tensor:
    """scores [B,Hkv,N] fp32 -> keep_idx [B,Hkv,budget] int32 ascending."""
    _require_cuda(scores)
    if scores.dtype != torch.float32 or scores.dim() != 3:
        raise ValueError("scores must be [B,Hkv,N] float32")
    B, Hkv, N = scores.shape
    if keep_idx is None:
        keep_idx = torch.empty((B, Hkv, max(int(budget), 0)), dtype=torch.int32, device=scores.device)
    elif keep_idx.dtype != torch.int32 or tuple(keep_idx.shape) != (B, Hkv, int(budget)) or not keep_idx.is_contiguous():
        raise ValueError("keep_idx must be a contiguous [B,Hkv,%d] int32 tensor" % int(budget))
    ws_ptr, ws_bytes, ws_hold = _select_ws(scores, workspace)
    rc = load_library().obc_select(scores.data_ptr(), int(budget), keep_idx.data_ptr(), B, Hkv, N,
                                   _lens_arg(seq_lens, B), ws_ptr, ws_bytes, _stream_ptr(scores))
    del ws_hold          # (released only now, after the kernels that use it were enqueued)
    if rc != OBC_OK:
        raise ObcError(rc, "obc_select")
    return keep_idx


def obc_select_protected(scores: torch.Tensor, num_hh: int, num_sinks: int = 0, num_recent: int = 0,
                         num_coming: int = 0, seq_lens=None, keep_idx: Optional[torch.Tensor] = None,
                         workspace=None) -> torch.Tensor:
    """scores [B,Hkv,N] fp32 -> keep_idx [B,Hkv,num_sinks+num_hh+num_recent-num_coming] int32 ascending."""
    _require_cuda(scores)
    if scores.dtype != torch.float32 or scores.dim() != 3:
        raise ValueError("scores must be [B,Hkv,N] float32")
    B, Hkv, N = scores.shape
    total = int(num_sinks) + int(num_hh) + int(num_recent) - int(num_coming)
    if keep_idx is None:
        keep_idx = torch.empty((B, Hkv, max(total, 0)), dtype=torch.int32, device=scores.device)
    elif keep_idx.dtype != torch.int32 or tuple(keep_idx.shape) != (B, Hkv, total) or not keep_idx.is_contiguous():
        raise ValueError("keep_idx must be a contiguous [B,Hkv,%d] int32 tensor" % total)
    ws_ptr, ws_bytes, ws_hold = _select_ws(scores, workspace)
    rc = load_library().obc_select_protected(scores.data_ptr(), int(num_hh), int(num_sinks), int(num_recent),
                                             int(num_coming), keep_idx.data_ptr(), B, Hkv, N,
                                             _lens_arg(seq_lens, B), ws_ptr, ws_bytes, _stream_ptr(scores))
    del ws_hold
    if rc != OBC_OK:
        raise ObcError(rc, "obc_select_protected")
    return keep_idx


def obc_select_pooled(scores: torch.Tensor, num_hh: int, pool: int = 5, num_sinks: int = 0, num_recent: int = 0,
                      num_coming: int = 0, seq_lens=None, keep_idx: Optional[torch.Tensor] = None,
                      workspace=None) -> torch.Tensor:
    """Like obc_select_protected, competitors ranked by their centred window sum of `pool` scores."""
    _require_cuda(scores)
    if scores.dtype != torch.float32 or scores.dim() != 3:
        raise ValueError("scores must be [B,Hkv,N] float32")
    B, Hkv, N = scores.shape
    total = int(num_sinks) + int(num_hh) + int(num_recent) - int(num_coming)
    if keep_idx is None:
        keep_idx = torch.empty((B, Hkv, max(total, 0)), dtype=torch.int32, device=scores.device)
    elif keep_idx.dtype != torch.int32 or tuple(keep_idx.shape) != (B, Hkv, total) or not keep_idx.is_contiguous():
        raise ValueError("keep_idx must be a contiguous [B,Hkv,%d] int32 tensor" % total)
    ws_ptr, ws_bytes, ws_hold = _select_ws(scores, workspace)
    rc = load_library().obc_select_pooled(scores.data_ptr(), int(num_hh), int(num_sinks), int(num_recent),
                                          int(num_coming), int(pool), keep_idx.data_ptr(), B, Hkv, N,
                                          _lens_arg(seq_lens, B), ws_ptr, ws_bytes, _stream_ptr(scores))
    del ws_hold
    if rc != OBC_OK:
        raise ObcError(rc, "obc_select_pooled")
    return keep_idx


def obc_select_adaptive(scores: torch.Tensor, budget: int, n_safe: int, cap: Optional[int] = None, seq_lens=None,
                        workspace: Optional[torch.Tensor] = None):
    """Head-adaptive budgets: (keep_idx [B,Hkv,cap] int32 ascending then -1, counts [B,Hkv] int32)."""
    _require_cuda(scores)
    if scores.dtype != torch.float32 or scores.dim() != 3:
        raise ValueError("scores must be [B,Hkv,N] float32")
    B, Hkv, N = scores.shape
    if cap is None:
        longest = N if seq_lens is None else max(int(x) for x in seq_lens)
        cap = min(longest, Hkv * int(budget) - (Hkv - 1) * int(n_safe))
    if workspace is None:
        need = ctypes.c_size_t(0)
        rc = load_library().obc_select_adaptive_workspace_bytes(B, Hkv, N, int(budget), int(n_safe), ctypes.byref(need))
        if rc != OBC_OK:
            raise ObcError(rc, "obc_select_adaptive_workspace_bytes")
        workspace = torch.empty(max(int(need.value), 256), dtype=torch.uint8, device=scores.device)
    keep_idx = torch.empty((B, Hkv, max(int(cap), 0)), dtype=torch.int32, device=scores.device)
    counts = torch.empty((B, Hkv), dtype=torch.int32, device=scores.device)
    rc = load_library().obc_select_adaptive(scores.data_ptr(), int(budget), int(n_safe), keep_idx.data_ptr(),
                                            counts.data_ptr(), int(cap), B, Hkv, N, _lens_arg(seq_lens, B),
                                            workspace.data_ptr(), workspace.numel(), _stream_ptr(scores))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_select_adaptive")
    return keep_idx, counts


def obc_compact(k: torch.Tensor, v: torch.Tensor, keep_idx: torch.Tensor, k_out=None, v_out=None):
    """k,v [B,Hkv,N,d], keep_idx [B,Hkv,budget] int32 -> (k_out, v_out) [B,Hkv,budget,d]."""
    _require_cuda(k, v, keep_idx)
    B, Hkv, N, d = k.shape
    budget = keep_idx.shape[-1]
    if keep_idx.dtype != torch.int32 or keep_idx.shape[:2] != (B, Hkv) or v.shape != k.shape:
        raise ValueError("keep_idx must be [B,Hkv,budget] int32 matching k, v")
    if k_out is None:
        k_out = torch.empty((B, Hkv, budget, d), dtype=k.dtype, device=k.device)
    if v_out is None:
        v_out = torch.empty((B, Hkv, budget, d), dtype=v.dtype, device=v.device)
    rc = load_library().obc_compact(k.data_ptr(), v.data_ptr(), keep_idx.data_ptr(), k_out.data_ptr(),
                                    v_out.data_ptr(), B, Hkv, N, budget, d, _dtype_code(k), _stream_ptr(k))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_compact")
    return k_out, v_out


def obc_compact_inplace(k: torch.Tensor, v: torch.Tensor, keep_idx: torch.Tensor,
                        scores: Optional[torch.Tensor] = None) -> None:
    """Moves rows keep_idx[b,g,j] of k, v (and entries of scores, whose tail is zeroed) to position j, in place."""
    _require_cuda(k, v, keep_idx)
    B, Hkv, N, d = k.shape
    budget = keep_idx.shape[-1]
    if keep_idx.dtype != torch.int32 or keep_idx.shape[:2] != (B, Hkv) or v.shape != k.shape:
        raise ValueError("keep_idx must be [B,Hkv,budget] int32 matching k, v")
    if not (k.is_contiguous() and v.is_contiguous() and keep_idx.is_contiguous()):
        raise ValueError("k, v and keep_idx must be contiguous")
    sp = None
    if scores is not None:
        _require_cuda(scores)
        if tuple(scores.shape) != (B, Hkv, N) or scores.dtype != torch.float32 or not scores.is_contiguous():
            raise ValueError("scores must be a contiguous [B,Hkv,N] float32 tensor")
        sp = scores.data_ptr()
    rc = load_library().obc_compact_inplace(k.data_ptr(), v.data_ptr(), sp, keep_idx.data_ptr(), B, Hkv, N, budget, d,
                                            _dtype_code(k), _stream_ptr(k))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_compact_inplace")


def obc_decode_step_workspace_bytes(B, N, Hq, Hkv, d, dtype, variant) -> int:
    out = ctypes.c_size_t(0)
    rc = load_library().obc_decode_step_workspace_bytes(B, N, Hq, Hkv, d, dtype, variant, ctypes.byref(out))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_decode_step_workspace_bytes")
    return int(out.value)


def obc_decode_step(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, scores: torch.Tensor, variant="joint",
                    num_sinks: int = 0, num_recent: int = 0, seq_lens=None, evicted: Optional[torch.Tensor] = None,
                    workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Accumulates the new row's scores, drops the lowest-scored unprotected token of every head and closes the gap in
    k, v and scores, all in place.  Returns the dropped positions [B,Hkv] int32."""
    _require_cuda(q, k, v, scores)
    B, Hq, W, d = q.shape
    _, Hkv, N, _ = k.shape
    if W != 1 or v.shape != k.shape or tuple(scores.shape) != (B, Hkv, N) or scores.dtype != torch.float32:
        raise ValueError("q must be [B,Hq,1,d], k, v [B,Hkv,N,d], scores [B,Hkv,N] float32")
    var = VARIANT_CODES[variant] if isinstance(variant, str) else int(variant)
    dt = _dtype_code(q)
    if workspace is None:
        workspace = torch.empty(obc_decode_step_workspace_bytes(B, N, Hq, Hkv, d, dt, var), dtype=torch.uint8, device=q.device)
    if evicted is None:
        evicted = torch.empty((B, Hkv), dtype=torch.int32, device=q.device)
    _require_cuda(evicted, workspace)
    rc = load_library().obc_decode_step(q.data_ptr(), k.data_ptr(), v.data_ptr(), scores.data_ptr(), evicted.data_ptr(), N,
                                        Hq, Hkv, d, var, B, dt, _lens_arg(seq_lens, B), int(num_sinks), int(num_recent),
                                        workspace.data_ptr(), workspace.numel(), _stream_ptr(q))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_decode_step")
    return evicted


def obc_compact_scores(scores: torch.Tensor, keep_idx: torch.Tensor, n_out: Optional[int] = None,
                       scores_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """scores [B,Hkv,N] fp32, keep_idx [B,Hkv,budget] -> [B,Hkv,n_out]: gathered scores, then zeros."""
    _require_cuda(scores, keep_idx)
    B, Hkv, N = scores.shape
    budget = keep_idx.shape[-1]
    if scores.dtype != torch.float32 or keep_idx.dtype != torch.int32 or tuple(keep_idx.shape[:2]) != (B, Hkv):
        raise ValueError("scores must be [B,Hkv,N] float32 and keep_idx [B,Hkv,budget] int32")
    n_out = budget if n_out is None else int(n_out)
    if scores_out is None:
        scores_out = torch.empty((B, Hkv, n_out), dtype=torch.float32, device=scores.device)
    elif tuple(scores_out.shape) != (B, Hkv, n_out) or scores_out.dtype != torch.float32 or not scores_out.is_contiguous():
        raise ValueError("scores_out must be a contiguous [B,Hkv,%d] float32 tensor" % n_out)
    rc = load_library().obc_compact_scores(scores.data_ptr(), keep_idx.data_ptr(), scores_out.data_ptr(), B, Hkv, N,
                                           budget, n_out, _stream_ptr(scores))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_compact_scores")
    return scores_out


OBC_PROBE_BLOCKS = 2048


def obc_probe_read_bandwidth(buf: torch.Tensor, sink: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Measurement hook: one streaming read of `buf` (time it with events around the call)."""
    if sink is None:
        sink = torch.empty(OBC_PROBE_BLOCKS * 256, dtype=torch.int32, device=buf.device)
    nbytes = buf.numel() * buf.element_size()
    rc = load_library().obc_probe_read_bandwidth(buf.data_ptr(), nbytes, sink.data_ptr(), _stream_ptr(buf))
    if rc != OBC_OK:
        raise ObcError(rc, "obc_probe_read_bandwidth")
    return sink
