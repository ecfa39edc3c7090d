"""Python binding of libs1f.so: segment-wise causal attention for sequence-level 1F1B (Seq1F1B,
arXiv 2406.03488) on MI355X.

Argument marshalling only: every step runs in the library's HIP kernels.  PyTorch supplies device
memory and the current stream.  There is no fallback: if the shared library is missing, importing the
compute entry points raises.
"""
from .binding import (COST_ADDITIVE, COST_LITERAL, Desc, S1FError, bwd_workspace_bytes, fwd_workspace_bytes,
                      kv_append, kv_grad_emit, seg_attn_fwd_ws,
                      library_path, load_library, partition, partition_ex, partition_rebalance, pipeline_simulate,
                      seq1f1b_interleaved_order, seq1f1b_interleaved_warmup, seg_attn_bwd, seg_attn_bwd_dkdv, seg_attn_bwd_dq,
                      seg_attn_bwd_noalloc, seg_attn_fwd, seq1f1b_order, seq1f1b_peak_memory_share, static_scratch_rows,
                      seq1f1b_warmup, strerror, version)

__all__ = ["COST_ADDITIVE", "COST_LITERAL", "Desc", "S1FError", "bwd_workspace_bytes", "fwd_workspace_bytes",
           "kv_append", "kv_grad_emit", "seg_attn_fwd_ws",
           "library_path", "load_library", "partition", "partition_ex", "partition_rebalance", "pipeline_simulate",
           "seq1f1b_interleaved_order", "seq1f1b_interleaved_warmup",
           "seg_attn_bwd", "seg_attn_bwd_dkdv", "seg_attn_bwd_dq", "seg_attn_bwd_noalloc", "seg_attn_fwd",
           "static_scratch_rows", "seq1f1b_order", "seq1f1b_peak_memory_share", "seq1f1b_warmup",
           "strerror", "version"]
