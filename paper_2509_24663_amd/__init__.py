"""MI355X (gfx950) implementation of InfLLM-V2's dense-sparse switchable attention.

The work is done by hand-written HIP kernels behind the C ABI declared in
``include/infllmv2.h`` (built into ``libinfllmv2.so`` next to this file).  This package is
only a thin ctypes binding with the same function names: it marshals torch tensors
(device memory, streams) into pointers and sizes.  There is no CPU fallback: if the
library has not been built, importing the binding raises.
"""
from . import binding as _binding
from .binding import (  # noqa: F401
    BF16,
    DecodeInfo,
    FP32,
    InfllmV2Error,
    Params,
    SeqInfo,
    block_scores,
    block_scores_pooled,
    compress_k,
    compress_k_append,
    decode_workspace_bytes,
    dense_attn_fwd,
    lib,
    num_cmp,
    sparse_attn_bwd,
    sparse_attn_fwd,
    sparse_decode,
    sparse_decode_static,
    sparse_decode_static_capacity,
    sparse_prefill,
    status_string,
    topk_blocks,
    topk_pooled,
    version,
    workspace_bytes,
)

# `op` codes of infllmv2_workspace_bytes
(OP_COMPRESS_K, OP_BLOCK_SCORES, OP_TOPK_BLOCKS, OP_SPARSE_ATTN_FWD, OP_DENSE_ATTN_FWD, OP_SPARSE_DECODE,
 OP_BLOCK_SCORES_POOLED, OP_TOPK_POOLED, OP_SPARSE_ATTN_BWD, OP_SPARSE_ATTN_BWD_MIN, OP_COMPRESS_K_APPEND) = (
    _binding.OP_COMPRESS_K, _binding.OP_BLOCK_SCORES, _binding.OP_TOPK_BLOCKS, _binding.OP_SPARSE_ATTN_FWD,
    _binding.OP_DENSE_ATTN_FWD, _binding.OP_SPARSE_DECODE, _binding.OP_BLOCK_SCORES_POOLED, _binding.OP_TOPK_POOLED,
    _binding.OP_SPARSE_ATTN_BWD, _binding.OP_SPARSE_ATTN_BWD_MIN, _binding.OP_COMPRESS_K_APPEND)
