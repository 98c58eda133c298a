"""kvp: block-wise prefill with a fixed-budget KV cache on AMD MI355X.

The work is done by libkvp.so (HIP kernels behind a C ABI, see include/kvp.h).
This package only marshals arguments; it has no fallback path.
"""
from .binding import (  # noqa: F401
    KVP_OK, KVP_EINVAL, KVP_ESTATE, KVP_ENOMEM, KVP_EDEVICE, KVP_TEXT, KVP_VISUAL,
    KVP_FLAG_DRY_RUN, KERNEL_KINDS, KvpError, KvpConfig, KvpSegment, KvpView, KvpKernelStat,
    lib, library_path, declared_symbols,
    kvp_strerror, kvp_cache_bytes, kvp_persistent_bytes, kvp_init_cache, kvp_prefill_chunk,
    kvp_prefill_chunk_proxy, kvp_prefill_chunk_keydiff, kvp_prefill_block, kvp_prefill_join,
    KVP_SCORE_OWN, KVP_SCORE_PROXY, KVP_SCORE_KEYDIFF,
    kvp_compact, kvp_compact_layers, kvp_set_deferred_scoring, kvp_decode_step, kvp_decode_step_static, KVP_STATIC_SCRATCH_BYTES, KVP_STATIC_MIN_SPLITS,
    kvp_decode_ready, kvp_set_state, kvp_set_attention_shape, kvp_set_score_sweep, kvp_debug_last,
    kvp_profile_enable,
    kvp_profile_read, kvp_kernel_name, kvp_debug_totals, TOTALS, kvp_probe_mfma, kvp_probe_copy, kvp_free_cache,
    Cache,
)
from .runtime import Prefill, LayerwisePrefill  # noqa: F401
