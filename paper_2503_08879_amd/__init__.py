"""MI355X-native SAGE-KV hot path: eviction pass + decode attention over the reduced cache.

`binding` wraps the C ABI declared in include/sagekv.h (and the measurement aids of
include/sagekv_bench.h) one to one.  Importing this package does
not load the library; the first call does, and raises if it was not built.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    BF16, F32, GROUP_SUM, PER_QUERY, SELECT_DENSE, DecodeDesc, PagedKV, SagekvError, SelectDesc, decode_desc, paged_select_desc,
    compact_pages, sagekv_append, sagekv_decode_attn_paged, sagekv_decode_step_paged, sagekv_select_into_pages,
    sagekv_paper_budget,
    sagekv_decode_attn, sagekv_decode_attn_window, sagekv_decode_step, sagekv_decode_step_ring, sagekv_decode_step_static, sagekv_decode_step_window, sagekv_decode_workspace_bytes,
    sagekv_select, sagekv_select_paged, sagekv_select_redone_rows, sagekv_select_workspace_bytes, sagekv_stage_timing_enable, sagekv_stage_timing_read, sagekv_stage_timing_stages,
    select_desc,
)
