"""Stateful token-reduced prefill of one hybrid (Mamba-2 / attention) layer on MI355X.

The work is done by hand-written HIP kernels behind the C ABI declared in
``include/strd.h``; this package is the thin binding (argument marshalling only).
"""
from .binding import (  # noqa: F401
    LIB_PATH, StrdError, attn_prefill, compact, compact_batch, lib, schedule_budgets, schedule_sigmoid,
    linear, linear_mfma, linear_library, linear_mfma_supported, rmsnorm, gated_rmsnorm, conv1d_silu, softplus_dt, avgpool, ssd_decode_step, attn_decode_step,
    schedule_step_decay, schedule_named, hybrid_layout, HYBRID_LAYERS, LAYER_MAMBA, LAYER_MLP, LAYER_ATTN, NAMED_SCHEDULES,
    score_attn, score_mamba, score_mamba_full, select_topk, ssd_prefill, ssd_prefill_gather,
    select_topk_noalloc, kernel_path, PATH_NONE, PATH_MFMA, PATH_SIMT,
    score_attn_varlen, score_mamba_varlen, select_topk_varlen, compact_varlen, mfma_rate_probe,
)

__all__ = [
    "LIB_PATH", "StrdError", "lib", "score_attn", "score_mamba", "score_mamba_full", "select_topk", "compact", "compact_batch",
    "ssd_prefill", "ssd_prefill_gather", "attn_prefill", "schedule_budgets", "schedule_sigmoid", "schedule_step_decay",
    "linear", "linear_mfma", "linear_library", "linear_mfma_supported", "rmsnorm", "gated_rmsnorm", "conv1d_silu", "softplus_dt", "avgpool", "ssd_decode_step", "attn_decode_step",
    "score_attn_varlen", "score_mamba_varlen", "select_topk_varlen", "compact_varlen", "mfma_rate_probe",
    "select_topk_noalloc", "kernel_path", "PATH_NONE", "PATH_MFMA", "PATH_SIMT", "schedule_named", "hybrid_layout", "HYBRID_LAYERS", "LAYER_MAMBA", "LAYER_MLP", "LAYER_ATTN", "NAMED_SCHEDULES",
]
