"""Seeded synthetic inputs for the InfLLM-V2 attention hot path.

This package holds no arithmetic of the method itself: it only draws random
Q/K/V with the shapes of the paper's model (Sec. 4.1: h_q 32, h_kv 2, d_h 128;
block size 64, compression 32/16) and a block-level "topic" structure so that
block scores are skewed the way real attention is.  Both the CPU oracle's tests
and the GPU tests / benchmark take their inputs from here, so the two sides see
the same bytes.
"""
from .generator import (  # noqa: F401
    CONFIGS,
    WorkloadConfig,
    bf16_bits,
    draw_ctx_lens,
    from_bf16_bits,
    make_config,
    make_decode,
    make_prefill,
    make_varlen,
    round_to_bf16,
)
