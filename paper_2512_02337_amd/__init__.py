"""SpecPV verification attention for MI355X: Python binding of libspecpv.so.

Argument marshalling only -- every step of the path runs in the HIP kernels
behind the C ABI declared in include/specpv.h.  torch is used for device memory
and streams.  There is no CPU fallback: if the HIP library is not built, load()
raises.
"""
from .binding import (REDUCE_LAST, REDUCE_MAX, REDUCE_MEAN, SCORE_EQ2, SCORE_CHANNEL_BOUND, SpecPVError, KV, Tree, SelectCfg, load,
                      lib_path, specpv_block_summarize, specpv_full_verify_refresh,
                      specpv_partial_verify_attn, specpv_select_blocks, specpv_workspace_bytes,
                      specpv_strerror, specpv_version, EXPORTS, MODE_FULL, MODE_PARTIAL, MODE_REFRESH,
                      specpv_select_mode, specpv_extend_parents, specpv_commit_accepted, specpv_commit_accepted_layers, specpv_gather_blocks,
                      specpv_partial_verify_attn_static, STATIC_SCRATCH_BYTES, specpv_debug_set_route, specpv_debug_set_select_route,
                      specpv_debug_set_timeline)

__all__ = ["REDUCE_LAST", "REDUCE_MAX", "REDUCE_MEAN", "SCORE_EQ2", "SCORE_CHANNEL_BOUND", "SpecPVError", "KV", "Tree", "SelectCfg", "load",
           "lib_path", "specpv_block_summarize", "specpv_full_verify_refresh", "specpv_partial_verify_attn",
           "specpv_select_blocks", "specpv_workspace_bytes", "specpv_strerror", "specpv_version", "EXPORTS",
           "MODE_FULL", "MODE_PARTIAL", "MODE_REFRESH", "specpv_select_mode", "specpv_extend_parents",
           "specpv_commit_accepted", "specpv_commit_accepted_layers", "specpv_gather_blocks",
           "specpv_partial_verify_attn_static", "STATIC_SCRATCH_BYTES", "specpv_debug_set_route", "specpv_debug_set_select_route",
           "specpv_debug_set_timeline"]
from .offload import LayerPrefetcher  # noqa: E402  (host-memory staging for the offloaded full cache)

__all__.append("LayerPrefetcher")
