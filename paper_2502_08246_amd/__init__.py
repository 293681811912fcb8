"""MI355X-native SAAP decode hot path (arXiv 2502.08246): thin Python binding over libsaap.so.

The package holds the HIP sources (csrc/), their build script and a ctypes binding whose
functions carry the names of the C entry points.  Every step runs in the HIP kernels; torch
is used for device memory and streams only.  There is no CPU fallback: calling an operation
without the built library or without a GPU raises.
"""
from .binding import (  # noqa: F401
    BF16, F32, GROUP_SUM, INDEPENDENT, LOGITS, PROBS, SaapError,
    adam_update, append_keys, assign_keys, bucket_attention_mass, bucket_attention_mass_batch, build_bucket_index, build_windowed_index, classify_queries, dense_decode_attention,
    dense_decode_attention_fp8, quantize_kv, query_model_loss_grads, query_model_bn_loss_grads, fold_batch_norm, sparse_decode_attention_fp8,
    library_path, lloyd_iterations, load_library, recompact_index, select_buckets, select_buckets_from_logits, sparse_decode_attention, stream_read_probe, mfma_rate_probe, update_centroids, window_push, window_push_fp8, append_keys_fp8, windowed_decode_attention, windowed_decode_attention_fp8,
    build_visit_plan, planned_decode_attention, planned_decode_attention_fp8, select_buckets_planned, visit_plan_ints, sparse_decode_attention_noalloc, prefill_sparse_attention, classify_select, select_attend, select_attend_fp8,
    workspace,
    workspace_bytes,
    workspace_reset,
)
