"""Thin ctypes binding of libsagekv.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels.  torch is used for device
memory (tensors are passed as raw device pointers) and for the current stream handle.
The binding fails loudly when the built library is missing; there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsagekv.so")

BF16, F32 = 0, 1
GROUP_SUM, PER_QUERY = 0, 1
STAGES = ("sample", "score", "stats", "combine", "topk", "redo", "gather")
SELECT_DENSE = 1

EXPORTS = (
    "sagekv_status_string", "sagekv_select_workspace_bytes", "sagekv_select", "sagekv_select_paged",
    "sagekv_select_redone_rows",
    "sagekv_append",
    "sagekv_decode_workspace_bytes", "sagekv_decode_attn", "sagekv_decode_step", "sagekv_decode_step_ring",
    "sagekv_decode_step_static",
    "sagekv_select_into_pages", "sagekv_decode_attn_paged", "sagekv_decode_step_paged",
    "sagekv_decode_attn_window", "sagekv_decode_step_window",
    "sagekv_stage_timing_enable", "sagekv_stage_timing_read", "sagekv_stage_timing_stages",
    "sagekv_paper_budget",
)


class SelectDesc(ctypes.Structure):
    _fields_ = [
        ("n_problems", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("head_mode", ctypes.c_int32),
        ("L", ctypes.c_int64),
        ("k_stride_problem", ctypes.c_int64), ("k_stride_head", ctypes.c_int64), ("k_stride_token", ctypes.c_int64),
        ("v_stride_problem", ctypes.c_int64), ("v_stride_head", ctypes.c_int64), ("v_stride_token", ctypes.c_int64),
        ("n_sink", ctypes.c_int32), ("n_recent", ctypes.c_int32), ("k", ctypes.c_int32),
        ("compact_capacity", ctypes.c_int32), ("flags", ctypes.c_uint32),
    ]


class PagedKV(ctypes.Structure):
    _fields_ = [
        ("block_table", ctypes.c_void_p), ("table_pitch", ctypes.c_int64), ("page_size", ctypes.c_int32),
        ("n_pages", ctypes.c_int32), ("k_stride_page", ctypes.c_int64), ("v_stride_page", ctypes.c_int64),
    ]


class DecodeDesc(ctypes.Structure):
    _fields_ = [
        ("n_problems", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int32), ("head_mode", ctypes.c_int32),
        ("n_sink", ctypes.c_int32), ("k", ctypes.c_int32), ("n_recent", ctypes.c_int32),
        ("compact_capacity", ctypes.c_int32), ("grow_recent", ctypes.c_int32),
    ]


class SagekvError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {status_string(code)} (status {code})")
        self.code = code


_lib = None


def lib():
    """The loaded library.  Raises if it has not been built (run __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2503_08879_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        L.sagekv_paper_budget.restype = ctypes.c_int
        L.sagekv_paper_budget.argtypes = [i32, i32, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.sagekv_status_string.restype = ctypes.c_char_p
        L.sagekv_status_string.argtypes = [ctypes.c_int]
        L.sagekv_select_workspace_bytes.restype = sz
        L.sagekv_select_workspace_bytes.argtypes = [ctypes.POINTER(SelectDesc)]
        L.sagekv_select.restype = ctypes.c_int
        L.sagekv_select.argtypes = [ctypes.POINTER(SelectDesc), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.sagekv_select_paged.restype = ctypes.c_int
        L.sagekv_select_paged.argtypes = [ctypes.POINTER(SelectDesc), ctypes.POINTER(PagedKV), vp, vp, vp, vp, vp, vp, vp,
                                          vp, sz, vp]
        L.sagekv_select_redone_rows.restype = ctypes.c_int
        L.sagekv_select_redone_rows.argtypes = [ctypes.POINTER(SelectDesc), vp, sz, vp, ctypes.POINTER(i32)]
        L.sagekv_append.restype = ctypes.c_int
        L.sagekv_append.argtypes = [ctypes.POINTER(DecodeDesc), vp, vp, vp, vp, i32, vp]
        L.sagekv_decode_workspace_bytes.restype = sz
        L.sagekv_decode_workspace_bytes.argtypes = [ctypes.POINTER(DecodeDesc)]
        L.sagekv_decode_attn.restype = ctypes.c_int
        L.sagekv_decode_attn.argtypes = [ctypes.POINTER(DecodeDesc), vp, vp, vp, i32, vp, vp, sz, vp]
        L.sagekv_decode_step.restype = ctypes.c_int
        L.sagekv_decode_step.argtypes = [ctypes.POINTER(DecodeDesc), vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
        L.sagekv_decode_step_ring.restype = ctypes.c_int
        L.sagekv_decode_step_ring.argtypes = [ctypes.POINTER(DecodeDesc), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        pk = ctypes.POINTER(PagedKV)
        L.sagekv_select_into_pages.restype = ctypes.c_int
        L.sagekv_select_into_pages.argtypes = [ctypes.POINTER(SelectDesc), pk, pk, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.sagekv_decode_attn_paged.restype = ctypes.c_int
        L.sagekv_decode_attn_paged.argtypes = [ctypes.POINTER(DecodeDesc), pk, vp, vp, vp, i32, vp, vp, sz, vp]
        L.sagekv_decode_step_paged.restype = ctypes.c_int
        L.sagekv_decode_step_paged.argtypes = [ctypes.POINTER(DecodeDesc), pk, vp, vp, vp, vp, vp, i32, vp, vp, vp, sz, vp]
        L.sagekv_decode_step_static.restype = ctypes.c_int
        L.sagekv_decode_step_static.argtypes = [ctypes.POINTER(DecodeDesc), vp, vp, vp, vp, vp, i32, vp, vp]
        L.sagekv_decode_attn_window.restype = ctypes.c_int
        L.sagekv_decode_attn_window.argtypes = [ctypes.POINTER(DecodeDesc), vp, vp, vp, vp, i32, vp, vp, sz, vp]
        L.sagekv_decode_step_window.restype = ctypes.c_int
        L.sagekv_decode_step_window.argtypes = [ctypes.POINTER(DecodeDesc), vp, vp, vp, vp, vp, vp, i32, vp, vp, sz, vp]
        L.sagekv_stage_timing_enable.restype = ctypes.c_int
        L.sagekv_stage_timing_enable.argtypes = [i32]
        L.sagekv_stage_timing_stages.restype = ctypes.c_int
        L.sagekv_stage_timing_stages.argtypes = [ctypes.c_uint32, i32]
        L.sagekv_stage_timing_read.restype = ctypes.c_int
        L.sagekv_stage_timing_read.argtypes = [i32, i32, ctypes.POINTER(ctypes.c_float)]
        _lib = L
    return _lib


def sagekv_paper_budget(B: int, G: int):
    """(n_sink, k, n_recent) of the paper's budget split for PER_QUERY selection (App. A.2)."""
    s, k, r = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(lib().sagekv_paper_budget(B, G, ctypes.byref(s), ctypes.byref(k), ctypes.byref(r)), "sagekv_paper_budget")
    return s.value, k.value, r.value


def status_string(code: int) -> str:
    return lib().sagekv_status_string(code).decode()


def _ptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream():
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_of(t) -> int:
    import torch

    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported element type {t.dtype}")


def _check(code: int, what: str):
    if code != 0:
        raise SagekvError(code, what)


# ---------------------------------------------------------------------------------------- select
def select_desc(q_last, K, V, n_sink, n_recent, k, compact_capacity=None, head_mode=GROUP_SUM, flags=0) -> SelectDesc:
    """Descriptor for q_last [P,Hq,d] and K, V [P,Hkv,L,d] (any strides with a unit inner stride)."""
    P, Hq, d = q_last.shape
    _, Hkv, L, _ = K.shape
    assert K.stride(3) == 1 and V.stride(3) == 1 and q_last.is_contiguous()
    lists = Hq // Hkv if head_mode == PER_QUERY else 1
    cap = n_sink + lists * k + n_recent if compact_capacity is None else compact_capacity
    return SelectDesc(P, Hq, Hkv, d, _dtype_of(K), head_mode, L, K.stride(0), K.stride(1), K.stride(2),
                      V.stride(0), V.stride(1), V.stride(2), n_sink, n_recent, k, cap, flags)


def sagekv_select_workspace_bytes(desc: SelectDesc) -> int:
    return lib().sagekv_select_workspace_bytes(ctypes.byref(desc))


def sagekv_select(desc: SelectDesc, q_last, K, V, Kc, Vc, kept_idx, scores_out, workspace) -> None:
    """Enqueue the eviction pass on torch's current stream.  All tensors are caller-allocated."""
    code = lib().sagekv_select(ctypes.byref(desc), _ptr(q_last), _ptr(K), _ptr(V), _ptr(Kc), _ptr(Vc),
                               _ptr(kept_idx), _ptr(scores_out), _ptr(workspace),
                               0 if workspace is None else workspace.numel() * workspace.element_size(), _stream())
    _check(code, "sagekv_select")


def paged_select_desc(q_last, K_pool, V_pool, block_table, L, n_sink, n_recent, k, compact_capacity=None,
                      head_mode=GROUP_SUM, flags=0):
    """Descriptors for q_last [P,Hq,d], page pools K_pool, V_pool [n_pages, Hkv, page_size, d] (any strides
    with a unit inner stride) and block_table [P, pages_per_problem] int32.  Returns (SelectDesc, PagedKV)."""
    import torch

    P, Hq, d = q_last.shape
    n_pages, Hkv, page_size, _ = K_pool.shape
    assert K_pool.stride(3) == 1 and V_pool.stride(3) == 1 and q_last.is_contiguous()
    assert block_table.dtype == torch.int32 and block_table.shape[0] == P and block_table.stride(1) == 1
    lists = Hq // Hkv if head_mode == PER_QUERY else 1
    cap = n_sink + lists * k + n_recent if compact_capacity is None else compact_capacity
    desc = SelectDesc(P, Hq, Hkv, d, _dtype_of(K_pool), head_mode, L, 0, K_pool.stride(1), K_pool.stride(2),
                      0, V_pool.stride(1), V_pool.stride(2), n_sink, n_recent, k, cap, flags)
    pages = PagedKV(block_table.data_ptr(), block_table.stride(0), page_size, n_pages, K_pool.stride(0),
                    V_pool.stride(0))
    return desc, pages


def sagekv_select_paged(desc: SelectDesc, pages: PagedKV, q_last, K_pool, V_pool, Kc, Vc, kept_idx, scores_out,
                        workspace) -> None:
    """sagekv_select over a paged cache (block table + page pools)."""
    code = lib().sagekv_select_paged(ctypes.byref(desc), ctypes.byref(pages), _ptr(q_last), _ptr(K_pool), _ptr(V_pool),
                                     _ptr(Kc), _ptr(Vc), _ptr(kept_idx), _ptr(scores_out), _ptr(workspace),
                                     _ws_bytes(workspace), _stream())
    _check(code, "sagekv_select_paged")


def sagekv_select_redone_rows(desc: SelectDesc, workspace) -> int:
    """Rows of the last sagekv_select on this workspace that the dense path had to redo (-1: dense call)."""
    n = ctypes.c_int32(0)
    _check(lib().sagekv_select_redone_rows(ctypes.byref(desc), _ptr(workspace), _ws_bytes(workspace), _stream(),
                                           ctypes.byref(n)), "sagekv_select_redone_rows")
    return n.value


# ---------------------------------------------------------------------------------------- decode
def decode_desc(n_problems, n_q_heads, n_kv_heads, head_dim, dtype, n_sink, k, n_recent, compact_capacity,
                grow_recent=False, head_mode=GROUP_SUM) -> DecodeDesc:
    return DecodeDesc(n_problems, n_q_heads, n_kv_heads, head_dim, dtype, head_mode, n_sink, k, n_recent,
                      compact_capacity, int(grow_recent))


def sagekv_decode_workspace_bytes(desc: DecodeDesc) -> int:
    return lib().sagekv_decode_workspace_bytes(ctypes.byref(desc))


def _ws_bytes(ws):
    return 0 if ws is None else ws.numel() * ws.element_size()


def sagekv_append(desc: DecodeDesc, k_new, v_new, Kc, Vc, n_appended: int) -> None:
    _check(lib().sagekv_append(ctypes.byref(desc), _ptr(k_new), _ptr(v_new), _ptr(Kc), _ptr(Vc), n_appended,
                               _stream()), "sagekv_append")


def sagekv_decode_attn(desc: DecodeDesc, q, Kc, Vc, length: int, out, workspace) -> None:
    _check(lib().sagekv_decode_attn(ctypes.byref(desc), _ptr(q), _ptr(Kc), _ptr(Vc), length, _ptr(out),
                                    _ptr(workspace), _ws_bytes(workspace), _stream()), "sagekv_decode_attn")


def sagekv_decode_step(desc: DecodeDesc, q, k_new, v_new, Kc, Vc, n_appended: int, out, workspace) -> None:
    _check(lib().sagekv_decode_step(ctypes.byref(desc), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(Kc), _ptr(Vc),
                                    n_appended, _ptr(out), _ptr(workspace), _ws_bytes(workspace), _stream()),
           "sagekv_decode_step")


def sagekv_decode_step_ring(desc: DecodeDesc, q, k_new, v_new, Kc, Vc, ring_state, out, workspace) -> None:
    """sagekv_decode_step with the append count in ring_state (device int32[2], zeroed by the caller)."""
    _check(lib().sagekv_decode_step_ring(ctypes.byref(desc), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(Kc), _ptr(Vc),
                                         _ptr(ring_state), _ptr(out), _ptr(workspace), _ws_bytes(workspace),
                                         _stream()), "sagekv_decode_step_ring")


def compact_pages(block_table, Kc_pool, Vc_pool) -> PagedKV:
    """Page description of a reduced cache: pools [n_pages, Hkv, page_size, d] (pages contiguous inside,
    any distance apart), block_table [P, pages_per_row] int32."""
    import torch

    n_pages, Hkv, page_size, d = Kc_pool.shape
    assert block_table.dtype == torch.int32 and block_table.stride(1) == 1
    for pool in (Kc_pool, Vc_pool):
        assert pool.stride(3) == 1 and pool.stride(2) == d and pool.stride(1) == page_size * d
    return PagedKV(block_table.data_ptr(), block_table.stride(0), page_size, n_pages, Kc_pool.stride(0), Vc_pool.stride(0))


def sagekv_select_into_pages(desc: SelectDesc, in_pages, out_pages: PagedKV, q_last, K, V, Kc_pool, Vc_pool, kept_idx,
                             scores_out, workspace) -> None:
    """The eviction pass gathering into a paged reduced cache (in_pages None: K, V strided)."""
    code = lib().sagekv_select_into_pages(ctypes.byref(desc), None if in_pages is None else ctypes.byref(in_pages),
                                          ctypes.byref(out_pages), _ptr(q_last), _ptr(K), _ptr(V), _ptr(Kc_pool),
                                          _ptr(Vc_pool), _ptr(kept_idx), _ptr(scores_out), _ptr(workspace),
                                          _ws_bytes(workspace), _stream())
    _check(code, "sagekv_select_into_pages")


def sagekv_decode_attn_paged(desc: DecodeDesc, pages: PagedKV, q, Kc_pool, Vc_pool, length: int, out, workspace) -> None:
    _check(lib().sagekv_decode_attn_paged(ctypes.byref(desc), ctypes.byref(pages), _ptr(q), _ptr(Kc_pool), _ptr(Vc_pool),
                                          length, _ptr(out), _ptr(workspace), _ws_bytes(workspace), _stream()),
           "sagekv_decode_attn_paged")


def sagekv_decode_step_paged(desc: DecodeDesc, pages: PagedKV, q, k_new, v_new, Kc_pool, Vc_pool, n_appended: int,
                             ring_state, out, workspace) -> None:
    _check(lib().sagekv_decode_step_paged(ctypes.byref(desc), ctypes.byref(pages), _ptr(q), _ptr(k_new), _ptr(v_new),
                                          _ptr(Kc_pool), _ptr(Vc_pool), n_appended, _ptr(ring_state), _ptr(out),
                                          _ptr(workspace), _ws_bytes(workspace), _stream()), "sagekv_decode_step_paged")


STATIC_SCRATCH_BYTES = 4 * 1024 * 1024
ERR_SCRATCH_LIMIT = 5


def sagekv_decode_step_static(desc: DecodeDesc, q, k_new, v_new, Kc, Vc, n_appended: int, out) -> None:
    """sagekv_decode_step on the library's built-in scratch: no workspace argument, no allocation."""
    _check(lib().sagekv_decode_step_static(ctypes.byref(desc), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(Kc), _ptr(Vc),
                                           n_appended, _ptr(out), _stream()), "sagekv_decode_step_static")


def sagekv_decode_attn_window(desc: DecodeDesc, q, q_sink, Kc, Vc, length: int, out, workspace) -> None:
    _check(lib().sagekv_decode_attn_window(ctypes.byref(desc), _ptr(q), _ptr(q_sink), _ptr(Kc), _ptr(Vc), length,
                                           _ptr(out), _ptr(workspace), _ws_bytes(workspace), _stream()),
           "sagekv_decode_attn_window")


def sagekv_decode_step_window(desc: DecodeDesc, q, q_sink, k_new, v_new, Kc, Vc, n_appended: int, out,
                              workspace) -> None:
    _check(lib().sagekv_decode_step_window(ctypes.byref(desc), _ptr(q), _ptr(q_sink), _ptr(k_new), _ptr(v_new),
                                           _ptr(Kc), _ptr(Vc), n_appended, _ptr(out), _ptr(workspace),
                                           _ws_bytes(workspace), _stream()), "sagekv_decode_step_window")


# ---------------------------------------------------------------------------------------- measurement aids
def sagekv_stage_timing_enable(n_calls: int) -> None:
    _check(lib().sagekv_stage_timing_enable(n_calls), "sagekv_stage_timing_enable")


def sagekv_stage_timing_stages(select_stages=None, decode: bool = True) -> None:
    """Which stages the timed calls bracket with events: a list of names from STAGES (None = all)."""
    mask = 0xFFFFFFFF if select_stages is None else sum(1 << STAGES.index(n) for n in select_stages)
    _check(lib().sagekv_stage_timing_stages(mask, int(decode)), "sagekv_stage_timing_stages")


def sagekv_stage_timing_read(which: int, call: int):
    buf = (ctypes.c_float * len(STAGES))()
    _check(lib().sagekv_stage_timing_read(which, call, buf), "sagekv_stage_timing_read")
    return list(buf) if which == 0 else [buf[0]]
