"""Transactional Attention KV-cache eviction pass, native on AMD gfx950.

The product is libta.so (HIP kernels behind the C ABI of include/ta.h); this
package is its thin Python binding plus the synthetic workload generators.
"""
from .binding import (DecodeState, EvictPlan, LayerEvictPlan, PagedKV, Params, TaError, layout_of, lib, ta_compact, ta_compact_into_pages, ta_decode_init, ta_decode_step,
                      ta_detect_anchors, ta_embed_anchors, ta_evict, ta_evict_layers, ta_evict_layers_paged, ta_evict_lse, ta_evict_paged, ta_evict_static, ta_expand_vouchers, ta_layer_budgets, ta_lookup_anchors,
                      ta_init, ta_match_anchors, ta_compact_paged, ta_score, ta_score_lse, ta_score_paged, ta_select, ta_workspace_bytes)

__all__ = ["DecodeState", "ta_decode_init", "ta_decode_step", "EvictPlan", "Params", "TaError", "layout_of", "lib", "ta_compact", "ta_compact_into_pages", "ta_evict", "ta_evict_lse", "ta_evict_paged", "ta_evict_static",
           "ta_evict_layers", "ta_evict_layers_paged", "LayerEvictPlan",
           "ta_detect_anchors", "ta_expand_vouchers", "ta_embed_anchors", "ta_lookup_anchors", "ta_layer_budgets",
           "ta_init", "ta_match_anchors", "ta_score", "ta_score_lse", "ta_score_paged", "ta_compact_paged", "PagedKV", "ta_select", "ta_workspace_bytes"]
