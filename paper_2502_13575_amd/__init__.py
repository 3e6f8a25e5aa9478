"""Python binding of libetsattn (decode attention over a tree-structured KV cache, gfx950).

Argument marshalling only: every step of the path runs in the HIP library.
There is no CPU fallback; loading fails loudly when the library is not built.
"""
from .binding import (ETS_BF16, ETS_F32, ETS_KV_FP8_E4M3, ETS_KV_NATIVE, ETS_PLAN_FLAT,
                      ETS_PLAN_TREE, ets_set_kv_format, ets_set_kv_head_scales, Context, EtsError,
                      EtsProfile, EtsShape, EtsStats, ets_create, ets_destroy, ets_plan, ets_plan_leaf_counts,
                      ets_plan_leaf_cover, ets_plan_paths, ets_plan_stats, ets_profile_read, ets_set_option,
                      ets_kv_append, ets_plan_advance, ets_plan_append_rows, ets_plan_check, ets_bench_read_stream, EtsPlanCheckReport, EtsPrefillStats, ets_plan_prefill,
                      ets_prefill_plan_stats, ets_prefill_q_ptr, ets_prefill_cover,
                      ets_tree_prefill_attn, EtsSelectInfo, ets_rebase_weights, ets_select_leaves,
                      ets_strerror, ets_tree_decode_attn, ets_tree_decode_attn_static,
                      ETS_STATIC_SCRATCH_BYTES, library_path, load_library)

__all__ = [
    "ETS_BF16", "ETS_F32", "ETS_KV_NATIVE", "ETS_KV_FP8_E4M3", "ets_set_kv_format", "ets_set_kv_head_scales",
    "ETS_PLAN_FLAT", "ETS_PLAN_TREE", "Context", "EtsError", "EtsShape",
    "EtsStats", "EtsProfile", "ets_profile_read", "ets_create", "ets_destroy", "ets_plan", "ets_plan_leaf_counts",
    "ets_plan_leaf_cover", "ets_plan_paths", "ets_plan_stats", "ets_set_option", "ets_strerror",
    "ets_kv_append", "ets_plan_advance", "ets_plan_append_rows", "ets_plan_check", "ets_bench_read_stream", "EtsPlanCheckReport", "EtsPrefillStats", "ets_plan_prefill",
    "ets_prefill_plan_stats", "ets_prefill_q_ptr", "ets_prefill_cover", "ets_tree_prefill_attn",
    "EtsSelectInfo", "ets_rebase_weights", "ets_select_leaves",
    "ets_tree_decode_attn", "ets_tree_decode_attn_static", "ETS_STATIC_SCRATCH_BYTES",
    "library_path", "load_library",
]
