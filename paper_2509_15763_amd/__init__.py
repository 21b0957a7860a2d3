"""libunigist: gist-masked causal attention (UniGist, Sec. 4.1-4.3) for MI355X.

All arithmetic runs in the HIP kernels of `libunigist.so`; this package only
marshals arguments (PyTorch supplies device memory and streams).  Importing the
package does not load the library; the first call does, and fails loudly if the
library has not been built.
"""
from .binding import (  # noqa: F401
    UNIGIST_BF16, UNIGIST_F32, UnigistError, lib_path, load,
    unigist_attn_fwd, unigist_attn_bwd, unigist_attn_bwd_stages, unigist_attn_bwd_workspace,
    BWD_STAGES, UNIGIST_BWD_ALL,
    unigist_decode, unigist_decode_workspace, unigist_decode_noalloc, unigist_decode_noalloc_scratch_bytes, unigist_debug_force_plain_alu, unigist_window_start,
    unigist_plan_row_tile, unigist_bwd_plan_build, unigist_plan_key_tile, unigist_plan_gist_unit, UNIGIST_WALK_FWD, UNIGIST_WALK_DQ,
    unigist_blockmap_build,
    unigist_status_str, unigist_tile_sizes, unigist_probe_mfma_rate, probe_mfma_rate, unigist_probe_read_rate, probe_read_rate,
    UNIGIST_E4M3, unigist_quantize_e4m3, unigist_decode_e4m3, quantize_e4m3, decode_e4m3,
    unigist_cache_update_ragged, unigist_prefill_chunk_ragged,
    unigist_prefill_chunk_e4m3, unigist_prefill_chunk_e4m3_workspace,
    unigist_attn_fwd_varlen_ex, unigist_attn_bwd_varlen_ex, unigist_attn_bwd_varlen_workspace_ex,
    unigist_prefill_chunk_view, unigist_prefill_chunk_strided, RingKVCache,
    unigist_attn_fwd_strided, unigist_attn_bwd_strided,
    unigist_attn_fwd_varlen_strided, unigist_attn_bwd_varlen_strided,
    unigist_cache_ring_rows, unigist_cache_to_ring, unigist_cache_from_ring, unigist_cache_ring_append,
    unigist_cache_rows, unigist_cache_update, unigist_prefill_chunk,
    UNIGIST_WINDOW_SLIDING, UNIGIST_WINDOW_UNITS,
    unigist_attn_fwd_ex, unigist_attn_bwd_ex, unigist_attn_bwd_workspace_ex, unigist_blockmap_build_ex,
    unigist_attn_fwd_varlen, unigist_attn_bwd_varlen, unigist_attn_bwd_varlen_workspace,
    attn_fwd_varlen, attn_bwd_varlen,
    unigist_cache_rows_ex, unigist_cache_update_ex, unigist_prefill_chunk_ex,
    attn_fwd, attn_bwd, decode, n_vis, KVCache, RaggedKVCache, prefill_chunk,
)
from .autograd import gist_attention, gist_attention_varlen  # noqa: F401,E402
