"""ctypes binding of oracle/obc_oracle.c (plain C, fp64).

Argument marshalling only; every formula lives in the C file, which cites the
paper passage it follows.  Inputs may be numpy arrays or CPU torch tensors of
any float dtype; they are upcast exactly to float64 before the call, so the
oracle sees the same bits (bf16 / fp32) the GPU path sees.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "obc_oracle.c")
_LIB = os.path.join(_HERE, "libobc_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over (batch, KV head)); returns the .so path."""
    with _lock:
        stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
        if force or stale:
            tmp = _LIB + ".tmp%d" % os.getpid()
            cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
                   "-ffp-contract=off", "-o", tmp, _SRC, "-lm"]
            subprocess.run(cmd, check=True)
            os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        path = build()
        lib = ctypes.CDLL(path)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        fp = ctypes.POINTER(ctypes.c_float)
        c_int = ctypes.c_int
        lib.obc_oracle_num_threads.restype = c_int
        lib.obc_oracle_window_attention.restype = c_int
        lib.obc_oracle_window_attention.argtypes = [dp, dp, dp] + [c_int] * 6 + [ip, dp, dp, dp]
        lib.obc_oracle_score.restype = c_int
        lib.obc_oracle_score.argtypes = [dp, dp, dp] + [c_int] * 6 + [ip, c_int, dp, dp, dp]
        lib.obc_oracle_attn_score.restype = c_int
        lib.obc_oracle_attn_score.argtypes = [dp, dp, dp] + [c_int] * 6 + [ip, dp]
        lib.obc_oracle_vatp_score.restype = c_int
        lib.obc_oracle_vatp_score.argtypes = lib.obc_oracle_attn_score.argtypes
        lib.obc_oracle_select.restype = c_int
        lib.obc_oracle_select.argtypes = [fp, c_int, c_int, c_int, c_int, ip, ip]
        lib.obc_oracle_select_protected.restype = c_int
        lib.obc_oracle_select_protected.argtypes = [fp, c_int, c_int, c_int, c_int, c_int, c_int, c_int, ip, ip]
        lib.obc_oracle_select_pooled.restype = c_int
        lib.obc_oracle_select_pooled.argtypes = [fp, c_int, c_int, c_int, c_int, c_int, c_int, c_int, c_int, ip, ip]
        lib.obc_oracle_select_adaptive.restype = c_int
        lib.obc_oracle_select_adaptive.argtypes = [fp, c_int, c_int, c_int, c_int, c_int, c_int, ip, ip, ip]
        lib.obc_oracle_compact.restype = c_int
        lib.obc_oracle_compact.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ip, c_int, c_int, c_int, c_int,
                                           ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().obc_oracle_num_threads())


def _f64(x) -> np.ndarray:
    if hasattr(x, "detach"):  # torch tensor (bf16 has no numpy dtype: go through float64)
        x = x.detach().cpu().double().numpy()
    return np.ascontiguousarray(x, dtype=np.float64)


def _dptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _lens(seq_lens, B):
    if seq_lens is None:
        return None, None
    a = np.ascontiguousarray(np.asarray(seq_lens, dtype=np.int32))
    if a.shape != (B,):
        raise ValueError("seq_lens must have B entries")
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _shapes(q, k, v):
    if q.ndim != 4 or k.ndim != 4 or v.shape != k.shape:
        raise ValueError("expected q [B,Hq,W,d], k,v [B,Hkv,N,d]")
    B, Hq, W, d = q.shape
    Bk, Hkv, N, dk = k.shape
    if Bk != B or dk != d:
        raise ValueError("q and k disagree on batch or head_dim")
    return B, Hq, Hkv, N, W, d


def _check(rc, what):
    if rc != 0:
        raise ValueError("%s: invalid arguments (code %d)" % (what, rc))


def window_attention(q, k, v, seq_lens=None):
    """Z, A [B,Hq,W,N] and O [B,Hq,W,d] of the window rows (small cases only)."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, Hq, Hkv, N, W, d = _shapes(q, k, v)
    keep, lp = _lens(seq_lens, B)
    Z = np.empty((B, Hq, W, N)); A = np.empty((B, Hq, W, N)); O = np.empty((B, Hq, W, d))
    rc = _load().obc_oracle_window_attention(_dptr(q), _dptr(k), _dptr(v), B, Hq, Hkv, N, W, d, lp,
                                             _dptr(Z), _dptr(A), _dptr(O))
    _check(rc, "window_attention")
    return Z, A, O


def score(q, k, v, seq_lens=None, joint_form: int = 0):
    """(S_value, S_key, S_joint), each [B,Hkv,N] float64."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, Hq, Hkv, N, W, d = _shapes(q, k, v)
    keep, lp = _lens(seq_lens, B)
    sv = np.empty((B, Hkv, N)); sk = np.empty((B, Hkv, N)); sj = np.empty((B, Hkv, N))
    rc = _load().obc_oracle_score(_dptr(q), _dptr(k), _dptr(v), B, Hq, Hkv, N, W, d, lp, int(joint_form),
                                  _dptr(sv), _dptr(sk), _dptr(sj))
    _check(rc, "score")
    return sv, sk, sj


def attn_score(q, k, v, seq_lens=None):
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, Hq, Hkv, N, W, d = _shapes(q, k, v)
    keep, lp = _lens(seq_lens, B)
    s = np.empty((B, Hkv, N))
    rc = _load().obc_oracle_attn_score(_dptr(q), _dptr(k), _dptr(v), B, Hq, Hkv, N, W, d, lp, _dptr(s))
    _check(rc, "attn_score")
    return s


def vatp_score(q, k, v, seq_lens=None):
    """sum_i |A_ip| * ||v_p||_1 per (b, KV head, token): the paper's reproduction of VATP."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, Hq, Hkv, N, W, d = _shapes(q, k, v)
    keep, lp = _lens(seq_lens, B)
    s = np.empty((B, Hkv, N))
    rc = _load().obc_oracle_vatp_score(_dptr(q), _dptr(k), _dptr(v), B, Hq, Hkv, N, W, d, lp, _dptr(s))
    _check(rc, "vatp_score")
    return s


def select(scores, budget: int, seq_lens=None):
    """keep_idx [B,Hkv,budget] int32 ascending from fp32 scores [B,Hkv,N]."""
    if hasattr(scores, "detach"):
        scores = scores.detach().cpu().numpy()
    s = np.ascontiguousarray(scores, dtype=np.float32)
    B, Hkv, N = s.shape
    keep, lp = _lens(seq_lens, B)
    out = np.empty((B, Hkv, budget), dtype=np.int32)
    rc = _load().obc_oracle_select(s.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), B, Hkv, N, int(budget), lp,
                                   out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    _check(rc, "select")
    return out


def select_protected(scores, num_hh: int, num_sinks: int = 0, num_recent: int = 0, num_coming: int = 0,
                     seq_lens=None):
    """keep_idx [B,Hkv,num_sinks+num_hh+num_recent-num_coming] int32 ascending (Algorithm 2 with sinks)."""
    if hasattr(scores, "detach"):
        scores = scores.detach().cpu().numpy()
    s = np.ascontiguousarray(scores, dtype=np.float32)
    B, Hkv, N = s.shape
    keep, lp = _lens(seq_lens, B)
    total = int(num_sinks) + int(num_hh) + int(num_recent) - int(num_coming)
    out = np.empty((B, Hkv, max(total, 0)), dtype=np.int32)
    rc = _load().obc_oracle_select_protected(s.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), B, Hkv, N,
                                             int(num_hh), int(num_sinks), int(num_recent), int(num_coming), lp,
                                             out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    _check(rc, "select_protected")
    return out


def select_pooled(scores, num_hh: int, pool: int = 5, num_sinks: int = 0, num_recent: int = 0, num_coming: int = 0,
                  seq_lens=None):
    """Like select_protected, with candidates ranked by their centred window sum of `pool` scores (fp32)."""
    if hasattr(scores, "detach"):
        scores = scores.detach().cpu().numpy()
    s = np.ascontiguousarray(scores, dtype=np.float32)
    B, Hkv, N = s.shape
    keep, lp = _lens(seq_lens, B)
    total = int(num_sinks) + int(num_hh) + int(num_recent) - int(num_coming)
    out = np.empty((B, Hkv, max(total, 0)), dtype=np.int32)
    rc = _load().obc_oracle_select_pooled(s.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), B, Hkv, N, int(num_hh),
                                          int(num_sinks), int(num_recent), int(num_coming), int(pool), lp,
                                          out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    _check(rc, "select_pooled")
    return out


def adaptive_cap(Hkv: int, budget: int, n_safe: int, max_len: int) -> int:
    """The most tokens one head can receive: everything beyond the other heads' safeguards."""
    return int(min(max_len, Hkv * budget - (Hkv - 1) * n_safe))


def select_adaptive(scores, budget: int, n_safe: int, cap=None, seq_lens=None):
    """(keep_idx [B,Hkv,cap] int32 ascending then -1, counts [B,Hkv] int32): head-adaptive budgets."""
    if hasattr(scores, "detach"):
        scores = scores.detach().cpu().numpy()
    s = np.ascontiguousarray(scores, dtype=np.float32)
    B, Hkv, N = s.shape
    keep, lp = _lens(seq_lens, B)
    if cap is None:
        cap = adaptive_cap(Hkv, budget, n_safe, N if seq_lens is None else max(seq_lens))
    out = np.empty((B, Hkv, max(int(cap), 0)), dtype=np.int32)
    counts = np.empty((B, Hkv), dtype=np.int32)
    rc = _load().obc_oracle_select_adaptive(s.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), B, Hkv, N, int(budget),
                                            int(n_safe), int(cap), lp,
                                            out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                            counts.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    _check(rc, "select_adaptive")
    return out, counts


def compact(k: np.ndarray, v: np.ndarray, keep_idx: np.ndarray):
    """Gather rows of k, v ([B,Hkv,N,d] numpy arrays of any fixed-size dtype) at keep_idx."""
    k = np.ascontiguousarray(k); v = np.ascontiguousarray(v)
    idx = np.ascontiguousarray(keep_idx, dtype=np.int32)
    B, Hkv, N, d = k.shape
    budget = idx.shape[-1]
    ko = np.empty((B, Hkv, budget, d), dtype=k.dtype); vo = np.empty_like(ko)
    rc = _load().obc_oracle_compact(k.ctypes.data, v.ctypes.data, idx.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                    B, Hkv, N, budget, d * k.dtype.itemsize, ko.ctypes.data, vo.ctypes.data)
    _check(rc, "compact")
    return ko, vo
