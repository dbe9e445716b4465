"""Seeded Q/K/V generator with block-topic structure (no method arithmetic here).

Recipe (per sequence, per KV head h):
  * every 64-token block j gets a topic vector  topic[h][j] ~ N(0, topic_std^2 I_d)
  * K[t, h] = N(0, I) + topic[h][t // 64]          V[t, h] = N(0, I)
  * every 64-token *query* block b picks one earlier block
        src[h][b] ~ Uniform{0 .. max(b - 1, 0)}
    and all G query heads of group h, for all tokens of that query block, get
        Q[t, g] = N(0, I) + topic_gain * topic[h][src[h][b]]
For bf16 workloads the values are rounded to bf16 (round-to-nearest-even) once,
here, so every consumer sees bf16-exact float32 numbers.

Layouts returned (float32 numpy arrays):
  q  [total_tokens, hq, d]      token-major, heads of one KV group contiguous
  k  [hkv, total_tokens, d]     head-major: a 64-token block is one contiguous run
  v  [hkv, total_tokens, d]
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

BASE_SEED = 20250924
TOPIC_BLOCK = 64


# --------------------------------------------------------------------------- bf16 helpers
def bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even, NaN kept quiet."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    out = (r >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        out = np.where(nan, np.uint16(0x7FC0), out)
    return out


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 and return them as float32."""
    return from_bf16_bits(bf16_bits(x)).reshape(x.shape)


# --------------------------------------------------------------------------- configs
@dataclass(frozen=True)
class WorkloadConfig:
    """One of the benchmark workloads: shapes plus method hyper-parameters."""

    name: str
    kind: str                      # "prefill" | "decode" | "varlen"
    dtype: str                     # "fp32" | "bf16"
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    seq_len: int = 0               # prefill
    lengths: Sequence[int] = ()    # varlen
    batch: int = 1                 # decode
    ctx_lo: int = 0                # decode: context lengths uniform in [ctx_lo, ctx_hi]
    ctx_hi: int = 0
    block_size: int = 64
    cmp_len: int = 32
    cmp_stride: int = 16
    pool_len: int = 5
    pool_stride: int = 4
    pool_pad: int = 0
    n_init: int = 1
    n_local: int = 8
    topk_total: int = 64
    dense_threshold: int = 0
    seed: int = BASE_SEED
    topic_std: float = 0.5

    @property
    def softmax_scale(self) -> float:
        return float(self.head_dim) ** -0.5

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads


CONFIGS: Dict[str, WorkloadConfig] = {
    "C1": WorkloadConfig("C1", "prefill", "fp32", 4, 1, 64, seq_len=2048, n_init=1, n_local=2,
                         topk_total=8, dense_threshold=1024, seed=BASE_SEED + 0),
    "C2": WorkloadConfig("C2", "prefill", "bf16", 32, 2, 128, seq_len=32768, seed=BASE_SEED + 1),
    "C3": WorkloadConfig("C3", "prefill", "bf16", 32, 2, 128, seq_len=131072, seed=BASE_SEED + 2),
    "C4": WorkloadConfig("C4", "decode", "bf16", 32, 2, 128, batch=16, ctx_lo=16384, ctx_hi=65536,
                         seed=BASE_SEED + 3),
    "C5": WorkloadConfig("C5", "varlen", "bf16", 32, 2, 128,
                         lengths=(512, 2048, 4096, 8192, 16384, 24576, 32768, 65536),
                         dense_threshold=8192, seed=BASE_SEED + 4),
}


# --------------------------------------------------------------------------- generators
def _normal(rng: np.random.Generator, shape) -> np.ndarray:
    return rng.standard_normal(shape, dtype=np.float32)


def _one_sequence(rng: np.random.Generator, n: int, hq: int, hkv: int, d: int,
                  topic_std: float, topic_gain: float, q_rows: Optional[np.ndarray] = None):
    """Draw one sequence.  q_rows: if given, only those token positions get a query row."""
    g = hq // hkv
    nb = (n + TOPIC_BLOCK - 1) // TOPIC_BLOCK
    topic = (topic_std * _normal(rng, (hkv, nb, d))).astype(np.float32)
    # src[h][b]: a uniformly chosen earlier block (block 0 and 1 both point at block 0)
    hi = np.maximum(np.arange(nb) - 1, 0)
    src = np.stack([rng.integers(0, hi + 1) for _ in range(hkv)]).astype(np.int64)   # [hkv, nb]
    blk = np.arange(n) // TOPIC_BLOCK
    k = _normal(rng, (hkv, n, d))
    k += topic[:, blk, :]
    v = _normal(rng, (hkv, n, d))
    pos = np.arange(n) if q_rows is None else np.asarray(q_rows, dtype=np.int64)
    q = _normal(rng, (len(pos), hq, d))
    qblk = pos // TOPIC_BLOCK
    for h in range(hkv):
        t = topic_gain * topic[h, src[h, qblk], :]                # [rows, d]
        q[:, h * g:(h + 1) * g, :] += t[:, None, :]
    return q, k, v, src


def _finish(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "fp32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(f"unknown dtype {dtype!r}")


def make_prefill(n: int, hq: int, hkv: int, d: int, *, seed: int, dtype: str = "bf16",
                 topic_std: float = 0.5, topic_gain: float = 1.0) -> dict:
    """One sequence of length n.  Returns q [n,hq,d], k/v [hkv,n,d], cu_seqlens, src."""
    rng = np.random.Generator(np.random.PCG64(seed))
    q, k, v, src = _one_sequence(rng, n, hq, hkv, d, topic_std, topic_gain)
    return dict(q=_finish(q, dtype), k=_finish(k, dtype), v=_finish(v, dtype),
                cu_seqlens=np.array([0, n], dtype=np.int32), src=[src], dtype=dtype)


def make_varlen(lengths: Sequence[int], hq: int, hkv: int, d: int, *, seed: int, dtype: str = "bf16",
                topic_std: float = 0.5, topic_gain: float = 1.0) -> dict:
    """Several independent sequences packed along the token axis (cu_seqlens marks the cuts)."""
    total = int(sum(lengths))
    q = np.empty((total, hq, d), dtype=np.float32)
    k = np.empty((hkv, total, d), dtype=np.float32)
    v = np.empty((hkv, total, d), dtype=np.float32)
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    srcs: List[np.ndarray] = []
    for i, n in enumerate(lengths):
        rng = np.random.Generator(np.random.PCG64([seed, i]))
        qi, ki, vi, si = _one_sequence(rng, int(n), hq, hkv, d, topic_std, topic_gain)
        a = int(cu[i])
        cu[i + 1] = a + int(n)
        q[a:a + n] = qi
        k[:, a:a + n] = ki
        v[:, a:a + n] = vi
        srcs.append(si)
    return dict(q=_finish(q, dtype), k=_finish(k, dtype), v=_finish(v, dtype),
                cu_seqlens=cu, src=srcs, dtype=dtype)


def make_decode(ctx_lens: Sequence[int], hq: int, hkv: int, d: int, *, seed: int, dtype: str = "bf16",
                topic_std: float = 0.5, topic_gain: float = 1.0, max_len: Optional[int] = None) -> dict:
    """Decode step: per sequence a K/V cache of ctx_lens[b] tokens (the new token's K/V already
    appended) and the one query row at position ctx_lens[b]-1.
    Returns q [batch,hq,d], k_cache/v_cache [batch,hkv,max_len,d] (zero beyond the context)."""
    ctx = np.asarray(ctx_lens, dtype=np.int32)
    b = len(ctx)
    lmax = int(max_len) if max_len is not None else int(ctx.max())
    q = np.empty((b, hq, d), dtype=np.float32)
    kc = np.zeros((b, hkv, lmax, d), dtype=np.float32)
    vc = np.zeros((b, hkv, lmax, d), dtype=np.float32)
    srcs = []
    for i in range(b):
        n = int(ctx[i])
        rng = np.random.Generator(np.random.PCG64([seed, i]))
        qi, ki, vi, si = _one_sequence(rng, n, hq, hkv, d, topic_std, topic_gain, q_rows=np.array([n - 1]))
        q[i] = qi[0]
        kc[i, :, :n] = ki
        vc[i, :, :n] = vi
        srcs.append(si)
    return dict(q=_finish(q, dtype), k_cache=_finish(kc, dtype), v_cache=_finish(vc, dtype),
                ctx_lens=ctx, src=srcs, dtype=dtype)


def draw_ctx_lens(batch: int, lo: int, hi: int, seed: int) -> np.ndarray:
    """Integer-uniform context lengths in [lo, hi] for the decode workload."""
    rng = np.random.Generator(np.random.PCG64([seed, 0xC7]))
    return rng.integers(lo, hi + 1, size=batch).astype(np.int32)


def make_config(cfg: WorkloadConfig, **overrides) -> dict:
    """Inputs for one of CONFIGS (optionally with a smaller seq_len / batch for tests)."""
    if cfg.kind == "prefill":
        n = overrides.get("seq_len", cfg.seq_len)
        return make_prefill(n, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, seed=cfg.seed,
                            dtype=cfg.dtype, topic_std=cfg.topic_std)
    if cfg.kind == "varlen":
        lens = overrides.get("lengths", cfg.lengths)
        return make_varlen(lens, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, seed=cfg.seed,
                           dtype=cfg.dtype, topic_std=cfg.topic_std)
    if cfg.kind == "decode":
        ctx = overrides.get("ctx_lens")
        if ctx is None:
            ctx = draw_ctx_lens(overrides.get("batch", cfg.batch), cfg.ctx_lo, cfg.ctx_hi, cfg.seed)
        return make_decode(ctx, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, seed=cfg.seed,
                           dtype=cfg.dtype, topic_std=cfg.topic_std)
    raise ValueError(cfg.kind)
