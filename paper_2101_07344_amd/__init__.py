"""Learned-cache lookup for AMD MI355X: thin Python binding over the C-ABI HIP library.

Everything the lookup computes runs in the hand-written kernels of ``libgati.so``;
this package only marshals arguments (PyTorch supplies device memory and streams).
There is no CPU or PyTorch fallback: if the library is missing, loading fails.
"""
from .binding import (  # noqa: F401
    GATI_OK, GATI_ERR_INVALID_ARG, GATI_ERR_UNSUPPORTED, GATI_ERR_OOM, GATI_ERR_DEVICE,
    GATI_F32, GATI_BF16, GATI_LAYOUT_NCS, GATI_LAYOUT_NSC, GATI_SEL_LINEAR, GATI_SEL_SOFTMAX, GATI_SEL_HIDDEN, GATI_PRED_GAP_MLP, GATI_PRED_POOL_FC, GATI_PRED_FC_MLP, GATI_PRED_CONV_FC, GATI_COMPACT_STATIC_MAX_ROWS,
    GatiError, CacheDesc, CacheWeights, TrainParams, Cache, CacheStack, Trainer,
    load_library, library_path, exported_symbols,
    gati_cache_create, gati_cache_destroy, gati_cache_lookup, gati_cache_lookup_compact, gati_cache_pool,
    gati_compact_misses, gati_compact_misses_static, gati_cache_set_selector, gati_cache_set_weights, gati_status_string, gati_cache_pool_variant,
    gati_trainer_create, gati_trainer_destroy, gati_trainer_step, gati_trainer_get_weights,
    gati_trainer_get_hidden_selector, gati_cache_load_trainer, gati_cache_fork, gati_probe_stream_read, gati_probe_copy, gati_probe_launch_chain,
)
