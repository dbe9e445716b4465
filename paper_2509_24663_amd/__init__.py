"""MI355X (gfx950) implementation of InfLLM-V2's dense-sparse switchable attention.

The work is done by hand-written HIP kernels behind the C ABI declared in
``include/infllmv2.h`` (built into ``libinfllmv2.so`` next to this file).  This package is
only a thin ctypes binding with the same function names: it marshals torch tensors
(device memory, streams) into pointers and sizes.  There is no CPU fallback: if the
library has not been built, importing the binding raises.
"""
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
    sparse_prefill,
    status_string,
    topk_blocks,
    topk_pooled,
    version,
)
