"""kvtrim: MI355X-native decode-time hot path of global retention-based KV eviction.

The work happens in libkvtrim.so (hand-written HIP for gfx950, C ABI declared in
include/kvtrim.h).  This package is the thin ctypes binding: same names as the
C entry points, argument marshalling only.  Importing it never loads the library;
the first call does, and fails loudly if it has not been built.
"""
from .binding import (PAGE_SIZE, Cache, Context, Gate, KvtrimError, PagedCache, kvtrim_gate_forward,
                      kvtrim_gate_forward_prepared, kvtrim_gate_prepare, kvtrim_gate_prepared_bytes,
                      kvtrim_gate_scratch_bytes, kvtrim_append, kvtrim_append_compact, kvtrim_compact,
                      kvtrim_compact_attn, kvtrim_compact_attn_inplace, kvtrim_compact_inplace, kvtrim_decode_attn, kvtrim_decode_attn_soft, kvtrim_kernel_name, kvtrim_min_room,
                      kvtrim_occupancy, kvtrim_paged_append, kvtrim_paged_attn, kvtrim_paged_build,
                      kvtrim_paged_defrag, kvtrim_paged_evict, kvtrim_paged_score, kvtrim_paged_score_select, kvtrim_paged_decode_step, kvtrim_paged_select, kvtrim_poll_error,
                      kvtrim_profile_begin, kvtrim_profile_end, kvtrim_score, kvtrim_select_global,
                      kvtrim_select_global_noalloc, kvtrim_score_select, kvtrim_select_path_counts, kvtrim_decode_step, kvtrim_decode_step_inplace,
                      kvtrim_workspace_bytes, library_path, load_library)

__all__ = ["PAGE_SIZE", "Cache", "Context", "Gate", "KvtrimError", "PagedCache", "kvtrim_gate_forward",
           "kvtrim_gate_forward_prepared", "kvtrim_gate_prepare", "kvtrim_gate_prepared_bytes",
           "kvtrim_gate_scratch_bytes", "kvtrim_append", "kvtrim_append_compact", "kvtrim_compact",
           "kvtrim_compact_attn", "kvtrim_compact_attn_inplace", "kvtrim_compact_inplace", "kvtrim_decode_attn", "kvtrim_decode_attn_soft", "kvtrim_kernel_name", "kvtrim_min_room",
           "kvtrim_occupancy", "kvtrim_paged_append", "kvtrim_paged_attn", "kvtrim_paged_build",
           "kvtrim_paged_defrag", "kvtrim_paged_evict", "kvtrim_paged_score", "kvtrim_paged_score_select", "kvtrim_paged_decode_step", "kvtrim_paged_select", "kvtrim_poll_error",
           "kvtrim_profile_begin", "kvtrim_profile_end", "kvtrim_score", "kvtrim_select_global",
           "kvtrim_select_global_noalloc", "kvtrim_score_select", "kvtrim_select_path_counts", "kvtrim_decode_step", "kvtrim_decode_step_inplace",
           "kvtrim_workspace_bytes", "library_path", "load_library"]
