"""MI355X-native PM-KVQ hot path: thin ctypes binding over libkvq.so (hand-written HIP for gfx950).

The binding marshals arguments only; every step of the path runs in the library's kernels.
Importing the package does not load the library; the first call does and raises if it is missing.
"""
from .binding import (  # noqa: F401
    KvqError, KvqConfig, KvqCache, load_library, library_path, exported_symbols,
    kvq_arena_bytes, kvq_bytes_per_token_head, kvq_status_string, kvq_calibrate_lambda, kvq_allocate_bits,
    kvq_decode_attention_batch, kvq_append_decode_attention_batch,
    KVQ_OK, KVQ_E_INVALID, KVQ_E_BUDGET, KVQ_E_OOM, KVQ_E_STATE, KVQ_E_HIP, KVQ_E_LIMIT,
    KVQ_POLICY_PAPER, KVQ_POLICY_OLDEST_FIRST, KVQ_WHICH_K, KVQ_WHICH_V,
    KVQ_OPT_SPLITS, KVQ_OPT_FUSED_MERGE, KVQ_OPT_DETERMINISTIC,
    KVQ_OPT_TILE_COST_2BIT, KVQ_OPT_TILE_COST_4BIT, KVQ_OPT_TILE_COST_8BIT, KVQ_OPT_TILE_COST_16BIT,
    KVQ_OPT_SHIFT_STRATEGY, KVQ_SHIFT_EQUIVALENT, KVQ_SHIFT_DIRECT, KVQ_SHIFT_MODIFIED,
    KVQ_OPT_TIER16, KVQ_TIER16_FP16, KVQ_TIER16_INT16,
)
