"""MI355X-native ZipVL prefill path: thin Python binding over libzipvl.so (C ABI).

Every step runs in the HIP kernels of the shared library; this package only
marshals arguments (device pointers, strides, the current HIP stream).  There
is no CPU fallback: calling any op without the built library raises.
"""
from .binding import (ZipvlError, library_path, load_library, dims_of, workspace_bytes,
                      zipvl_score, zipvl_score_all_rows, zipvl_select, zipvl_share_scores, zipvl_sparse_prefill, zipvl_compact_kv,
                      zipvl_kv_append, zipvl_decode_attn, zipvl_decode_attn_static, zipvl_decode_step, decode_step_workspace, select_workspace, zipvl_version, zipvl_last_error,
                      zipvl_quantize_kv, zipvl_decode_attn_q, QCache, QTensor,
                      OUT_FULL, OUT_COMPACT, KV_ALREADY_COMPACT, T_PER_BATCH, SCORE_PER_QHEAD,
                      SELECT_NEGATIVE, SELECT_NONFINITE, SELECT_OVERFLOW,
                      OP_SCORE, OP_SELECT, OP_SPARSE_PREFILL, OP_DECODE, OP_QUANTIZE_KV, OP_DECODE_Q, OP_SCORE_ALL_ROWS, OP_DECODE_STEP, EXPORTS,
                      KERNELS, zipvl_timing_enable, zipvl_timing_read, zipvl_probe_peaks)

__all__ = ["ZipvlError", "library_path", "load_library", "dims_of", "workspace_bytes",
           "zipvl_score", "zipvl_score_all_rows", "zipvl_select", "zipvl_share_scores", "zipvl_sparse_prefill", "zipvl_compact_kv",
           "zipvl_kv_append", "zipvl_decode_attn", "zipvl_decode_attn_static", "zipvl_decode_step", "decode_step_workspace", "select_workspace", "zipvl_version", "zipvl_last_error",
           "zipvl_quantize_kv", "zipvl_decode_attn_q", "QCache", "QTensor",
           "OUT_FULL", "OUT_COMPACT", "KV_ALREADY_COMPACT", "T_PER_BATCH", "SCORE_PER_QHEAD",
           "SELECT_NEGATIVE", "SELECT_NONFINITE", "SELECT_OVERFLOW",
           "OP_SCORE", "OP_SELECT", "OP_SPARSE_PREFILL", "OP_DECODE", "OP_QUANTIZE_KV", "OP_DECODE_Q", "OP_SCORE_ALL_ROWS", "OP_DECODE_STEP", "EXPORTS",
           "KERNELS", "zipvl_timing_enable", "zipvl_timing_read", "zipvl_probe_peaks"]
