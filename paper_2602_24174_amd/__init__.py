"""MI355X-native TASC-spec: n-gram-drafted greedy speculative decoding (HIP kernels behind a C ABI).

The package holds the HIP sources (csrc/), their build script and a thin ctypes binding whose functions
carry the names of the C entry points declared in include/tasc.h.
"""
from .binding import (  # noqa: F401
    EXPORTS, LIB_PATH, TascError, GenStats, ModelDesc, NgramStats, SpecParams, WeightPtrs, lib, spec_params,
    tasc_draft, tasc_generate, tasc_session_status, tasc_profile_enable, tasc_calibration_copy, tasc_calibration_mfma, tasc_calibration_read, tasc_calibration_handover, tasc_calibration_gemm, tasc_profile_phases, tasc_config_set, TASC_CFG_SMALL_PATH, TASC_CFG_SMALL_GRID, TASC_CFG_SMALL_LAYER_WGS, TASC_CFG_SMALL_LAYER_STRIDE, TASC_CFG_TILED_PATH, TASC_CFG_SMALL_XCD_LOCAL, TASC_CFG_SMALL_LAYER_WORKERS, TASC_CFG_SMALL_KERNEL, TASC_CFG_PIPE_SHARE, TASC_CFG_CHAINS, TASC_CFG_STEP_GRAPH, tasc_profile_read, tasc_profile_durations, KERNEL_CLASSES, tasc_model_create, tasc_ngram_build, tasc_ngram_export, tasc_ngram_export_contexts,
    tasc_ngram_get_stats, tasc_model_bigram, tasc_ngram_from_bigram, tasc_tok_enrich, tasc_ngram_entropy, tasc_ngram_entropy_noalloc, TableEntropy, tasc_ngram_unigram, tasc_session_create, tasc_session_get_tokens, tasc_session_kv_bytes,
    tasc_session_prefill, tasc_session_workspace_bytes, tasc_verify_step,
)
