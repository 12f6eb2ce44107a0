"""MI355X-native Kwai Summary Attention hot path: ctypes binding of libksa.so plus seeded input generators.

The native library is loaded on first use (binding.lib()); nothing here computes attention in Python.
"""
from .binding import (KSA_FLAG_SUMMARY_SELF_ONLY, KSA_ROW_SUMMARY, KSA_ROW_TEXT, KSA_SPACE_SUMMARY, KSA_SPACE_TEXT, KSA_TILE_FULL,
                      KSA_TILE_MASKED, KsaError, Layout, build_info, cache_geometry, cache_summary_row,
                      cache_text_row, decode_workspace_bytes, ksa_build_layout, ksa_cache_append,
                      ksa_cache_from_prefill, ksa_decode_fwd, ksa_decode_fwd_static, KSA_DECODE_STATIC_SCRATCH_BYTES, ksa_decode_ranges, ksa_decode_summary_fwd,
                      ksa_decode_summary_ranges, ksa_params, ksa_prefill_bwd, ksa_prefill_fwd, ksa_prefill_relayout_v, make_params,
                      pack_cache, prefill_bwd_workspace_bytes, prefill_workspace_bytes)

__all__ = ["KSA_FLAG_SUMMARY_SELF_ONLY", "KSA_ROW_SUMMARY", "KSA_ROW_TEXT", "KSA_SPACE_SUMMARY", "KSA_SPACE_TEXT", "KSA_TILE_FULL",
           "KSA_TILE_MASKED", "KsaError", "Layout", "build_info", "cache_geometry", "cache_summary_row",
           "cache_text_row", "decode_workspace_bytes", "ksa_build_layout", "ksa_cache_append",
           "ksa_cache_from_prefill", "ksa_decode_fwd", "ksa_decode_fwd_static", "KSA_DECODE_STATIC_SCRATCH_BYTES",
           "ksa_decode_ranges", "ksa_decode_summary_fwd",
           "ksa_decode_summary_ranges", "ksa_params", "ksa_prefill_bwd", "ksa_prefill_fwd", "ksa_prefill_relayout_v", "make_params",
           "pack_cache", "prefill_bwd_workspace_bytes", "prefill_workspace_bytes"]
