"""ctypes binding of the CPU oracle (`sagekv_ref.c`).

TEST INFRASTRUCTURE ONLY: imported by tests/, by `__graft_entry__.smoke()` and by
`bench.py`'s cpu_baseline leg; never by the product package.

Arrays are numpy, contiguous, element type uint16 (bf16 bit patterns, dtype=0) or
float32 (dtype=1).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sagekv_ref.c")
_LIB = os.path.join(_HERE, "libsagekv_ref.so")

BF16, F32 = 0, 1
GROUP_SUM, PER_QUERY = 0, 1


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", _SRC, "-o", _LIB, "-lm"]
        )
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        for name in ("sagekv_ref_scores", "sagekv_ref_select", "sagekv_ref_append", "sagekv_ref_decode_attn",
                     "sagekv_ref_decode_attn_window_rope", "sagekv_ref_full_attention", "sagekv_ref_threads"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def threads() -> int:
    return lib().sagekv_ref_threads()


def _p(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else ctypes.c_void_p(0)


def _check(a, dtype):
    want = np.uint16 if dtype == BF16 else np.float32
    assert a.dtype == want and a.flags.c_contiguous, (a.dtype, want)


def n_lists(head_mode, Hq, Hkv):
    return 1 if head_mode == GROUP_SUM else Hq // Hkv


def scores(dtype, head_mode, q_last, K):
    """q_last [P,Hq,d], K [P,Hkv,L,d] -> fp32 [P,Hkv,n_lists,L]."""
    _check(q_last, dtype), _check(K, dtype)
    P, Hq, d = q_last.shape
    _, Hkv, L, _ = K.shape
    out = np.empty((P, Hkv, n_lists(head_mode, Hq, Hkv), L), dtype=np.float32)
    rc = lib().sagekv_ref_scores(dtype, head_mode, P, Hq, Hkv, d, ctypes.c_int64(L), _p(q_last), _p(K), _p(out))
    if rc:
        raise ValueError(f"sagekv_ref_scores: {rc}")
    return out


def select(dtype, head_mode, q_last, K, V, S, W, k, cap=None, want_scores=False):
    """Eviction pass.  Returns (Kc, Vc, kept_idx[, scores])."""
    for a in (q_last, K, V):
        _check(a, dtype)
    P, Hq, d = q_last.shape
    _, Hkv, L, _ = K.shape
    nl = n_lists(head_mode, Hq, Hkv)
    n_kept = S + nl * k + W
    cap = n_kept if cap is None else cap
    Kc = np.zeros((P, Hkv, cap, d), dtype=K.dtype)
    Vc = np.zeros((P, Hkv, cap, d), dtype=K.dtype)
    kept = np.full((P, Hkv, max(n_kept, 0)), -1, dtype=np.int32)
    s = np.empty((P, Hkv, nl, L), dtype=np.float32) if want_scores else None
    rc = lib().sagekv_ref_select(dtype, head_mode, P, Hq, Hkv, d, ctypes.c_int64(L), S, W, k, cap, _p(q_last), _p(K),
                                 _p(V), _p(Kc), _p(Vc), _p(kept), _p(s))
    if rc:
        raise ValueError(f"sagekv_ref_select: {rc}")
    return (Kc, Vc, kept, s) if want_scores else (Kc, Vc, kept)


def append(dtype, Kc, Vc, k_new, v_new, seg, W, grow=False, length=0):
    """In place.  Returns the new length (grow) or `length` unchanged (fifo)."""
    for a in (Kc, Vc, k_new, v_new):
        _check(a, dtype)
    P, Hkv, cap, d = Kc.shape
    ln = ctypes.c_int32(length)
    rc = lib().sagekv_ref_append(dtype, P, Hkv, d, cap, seg, W, int(grow), ctypes.byref(ln), _p(k_new), _p(v_new),
                                 _p(Kc), _p(Vc))
    if rc:
        raise ValueError(f"sagekv_ref_append: {rc}")
    return ln.value


def decode_attn(dtype, head_mode, q, Kc, Vc, length, S=0, k=0, W=0):
    """q [P,Hq,d], Kc/Vc [P,Hkv,cap,d] -> out fp32 [P,Hq,d]."""
    for a in (q, Kc, Vc):
        _check(a, dtype)
    P, Hq, d = q.shape
    _, Hkv, cap, _ = Kc.shape
    out = np.empty((P, Hq, d), dtype=np.float32)
    rc = lib().sagekv_ref_decode_attn(dtype, head_mode, P, Hq, Hkv, d, cap, S, k, W, length, _p(q), _p(Kc), _p(Vc),
                                      _p(out))
    if rc:
        raise ValueError(f"sagekv_ref_decode_attn: {rc}")
    return out


def decode_attn_window_rope(dtype, q, Kc, Vc, length, inv_freq):
    """StreamLLM_R decode attention: un-rotated q [P,Hq,d] and Kc [P,Hkv,cap,d] (window order), rotary
    positions = window indices, query at length-1; inv_freq fp64 [d/2] -> out fp32 [P,Hq,d]."""
    for a in (q, Kc, Vc):
        _check(a, dtype)
    P, Hq, d = q.shape
    _, Hkv, cap, _ = Kc.shape
    f = np.ascontiguousarray(inv_freq, dtype=np.float64)
    assert f.shape == (d // 2,)
    out = np.empty((P, Hq, d), dtype=np.float32)
    rc = lib().sagekv_ref_decode_attn_window_rope(dtype, P, Hq, Hkv, d, cap, length, _p(q), _p(Kc), _p(Vc), _p(f),
                                                  _p(out))
    if rc:
        raise ValueError(f"sagekv_ref_decode_attn_window_rope: {rc}")
    return out


def full_attention(dtype, q, K, V, idx=None):
    """q [G,d], K/V [L,d] of ONE KV head -> out fp32 [G,d], attending all of [0,L) or the listed positions."""
    for a in (q, K, V):
        _check(a, dtype)
    G, d = q.shape
    L = K.shape[0]
    out = np.empty((G, d), dtype=np.float32)
    if idx is not None:
        idx = np.ascontiguousarray(idx, dtype=np.int64)
    rc = lib().sagekv_ref_full_attention(dtype, G, d, ctypes.c_int64(L), _p(q), _p(K), _p(V), _p(idx),
                                         ctypes.c_int64(0 if idx is None else len(idx)), _p(out))
    if rc:
        raise ValueError(f"sagekv_ref_full_attention: {rc}")
    return out


def paper_budget(B, G):
    s, k, r = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    lib().sagekv_ref_paper_budget(B, G, ctypes.byref(s), ctypes.byref(k), ctypes.byref(r))
    return s.value, k.value, r.value
