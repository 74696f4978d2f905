"""MI355X-native sparse attention for LongGen's efficient layers (arxiv 2410.01485).

Thin ctypes binding over liblonggen_attn.so (hand-written HIP for gfx950).  PyTorch is
used only for device memory and streams; every step of the path runs in the library.
"""
from .binding import (LG_BF16, LG_F32, LgError, bwd_varlen_workspace_bytes, bwd_workspace_bytes,
                      lg_sparse_attn_bwd_varlen, lg_sparse_attn_fwd_varlen, decode_cache_workspace_bytes,
                      decode_paged_workspace_bytes, decode_workspace_bytes, lg_kv_paged_append,
                      lg_sparse_attn_decode_paged, lg_debug_bwd_kernel_ms, lg_debug_decode_segments, lg_debug_decode_split_headdim, lg_debug_partial_tile_bits, lg_debug_pattern_fields, lg_debug_tile_map, lg_debug_tile_walk,
                      lg_kv_cache_slots, lg_kv_ring_append, lg_sparse_attn_bwd, lg_sparse_attn_decode,
                      lg_sparse_attn_decode_cache, lg_sparse_attn_decode_cache_static, lg_sparse_attn_fwd, lib, lib_path,
                      status_str)

__all__ = ["LG_BF16", "LG_F32", "LgError", "bwd_varlen_workspace_bytes", "bwd_workspace_bytes",
           "lg_sparse_attn_bwd_varlen", "lg_sparse_attn_fwd_varlen", "decode_cache_workspace_bytes",
           "decode_paged_workspace_bytes", "decode_workspace_bytes", "lg_kv_paged_append",
           "lg_sparse_attn_decode_paged", "lg_debug_bwd_kernel_ms", "lg_debug_decode_segments", "lg_debug_decode_split_headdim", "lg_debug_partial_tile_bits", "lg_debug_pattern_fields", "lg_debug_tile_map", "lg_debug_tile_walk",
           "lg_kv_cache_slots", "lg_kv_ring_append", "lg_sparse_attn_bwd", "lg_sparse_attn_decode",
           "lg_sparse_attn_decode_cache", "lg_sparse_attn_decode_cache_static", "lg_sparse_attn_fwd", "lib", "lib_path",
           "status_str"]
