"""CPU oracle of the InfLLM-V2 attention path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper over ``oracle.c`` (plain C, double arithmetic, OpenMP over
query rows) plus the compositions the paper describes in prose: varlen packing,
the dense/sparse switch (Sec. 3.2, last paragraph of "Aligned Computation") and
a decode step as the last row of a prefill.  Nothing in the GPU package imports
this module and this module imports nothing from the GPU package.

Only tests, the smoke check and the benchmark's cpu_baseline leg may use it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile oracle.c into liboracle.so next to it (gcc, -O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        i32, i64, f64 = ctypes.c_int, ctypes.c_int64, ctypes.c_double
        P = ctypes.c_void_p
        lib.oracle_num_cmp.restype = ctypes.c_int
        lib.oracle_num_cmp.argtypes = [i32, i32, i32]
        lib.oracle_visible_cmp.restype = ctypes.c_int
        lib.oracle_visible_cmp.argtypes = [i32, i32, i32]
        lib.oracle_compress_k.restype = None
        lib.oracle_compress_k.argtypes = [P, i32, i32, i32, i32, P]
        lib.oracle_block_scores.restype = None
        lib.oracle_block_scores.argtypes = [P, P, i32, i32, i32, P, i32, i32, i32, f64, P, i64]
        lib.oracle_block_scores_lse_approx.restype = None
        lib.oracle_block_scores_lse_approx.argtypes = [P, P, i32, i32, i32, P, i32, i32, i32, P, i32, i32, i32, f64, P, i64]
        lib.oracle_topk_blocks.restype = None
        lib.oracle_topk_blocks.argtypes = [P, i64, P, i32, i32, i32, i32, i32, i32, i32, i32, i32, i32, P, P, i64]
        lib.oracle_sparse_attn.restype = None
        lib.oracle_sparse_attn.argtypes = [P, P, i32, i32, i32, P, P, i32, i32, P, i32, f64, P, P]
        lib.oracle_dense_attn.restype = None
        lib.oracle_dense_attn.argtypes = [P, P, i32, i32, i32, P, P, i32, f64, P, P]
        lib.oracle_attn_bwd.restype = None
        lib.oracle_attn_bwd.argtypes = [P, P, i32, i32, i32, P, P, i32, i32, P, i32, f64, P, P, P, P]
        _lib = lib
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


@dataclass(frozen=True)
class Params:
    """Hyper-parameters of the method in the paper's notation (Sec. 3.2, 3.3, 4.1)."""

    block_size: int = 64        # B
    cmp_len: int = 32           # l_C1
    cmp_stride: int = 16        # s_C1
    pool_len: int = 5           # l
    pool_stride: int = 4        # s
    pool_pad: int = 0           # 0: window [s*j, s*j+l) exactly as printed in Eq. 6
    n_init: int = 1             # |I_init|
    n_local: int = 8            # |I_local|
    topk_total: int = 64        # |I|
    dense_threshold: int = 0    # sequences shorter than this run dense attention
    softmax_scale: float = 128 ** -0.5
    lse_mode: int = 0           # 1: LSE Approximation (Sec. 3.4): normalise with the log-sum-exp over K^{C2}

    @staticmethod
    def from_config(cfg) -> "Params":
        return Params(cfg.block_size, cfg.cmp_len, cfg.cmp_stride, cfg.pool_len, cfg.pool_stride, cfg.pool_pad,
                      cfg.n_init, cfg.n_local, cfg.topk_total, cfg.dense_threshold, cfg.softmax_scale)


# --------------------------------------------------------------------------- per-head steps
def num_cmp(n: int, p: Params) -> int:
    return _load().oracle_num_cmp(int(n), p.cmp_len, p.cmp_stride)


def visible_cmp(t: int, p: Params) -> int:
    return _load().oracle_visible_cmp(int(t), p.cmp_len, p.cmp_stride)


def compress_k(K: np.ndarray, p: Params, level: int = 1) -> np.ndarray:
    """Eq. 3 (level 1: K^{C1}) or Eq. 7 (level 2: K^{C2}, window and stride four times as long).
    K [n, d] (one KV head, one sequence) -> [nc, d]."""
    K = _f32(K)
    n, d = K.shape
    lc, sc = (p.cmp_len, p.cmp_stride) if level == 1 else (4 * p.cmp_len, 4 * p.cmp_stride)
    kc = np.zeros((_load().oracle_num_cmp(int(n), lc, sc), d), dtype=np.float32)
    _load().oracle_compress_k(_p(K), n, d, lc, sc, _p(kc))
    return kc


def block_scores(Q: np.ndarray, pos: np.ndarray, kc: np.ndarray, p: Params, kc2: Optional[np.ndarray] = None) -> np.ndarray:
    """Eq. 4-5.  Q [rows, G, d], pos [rows], kc [nc, d] -> S^shared [rows, nc].
    With p.lse_mode == 1 (LSE Approximation, Sec. 3.4) kc2 = K^{C2} [nc2, d] is required."""
    Q, pos, kc = _f32(Q), _i32(pos), _f32(kc)
    nr, G, d = Q.shape
    nc = kc.shape[0]
    out = np.zeros((nr, max(nc, 1)), dtype=np.float32)
    if p.lse_mode == 0:
        _load().oracle_block_scores(_p(Q), _p(pos), nr, G, d, _p(kc), nc, p.cmp_len, p.cmp_stride,
                                    float(p.softmax_scale), _p(out), out.shape[1])
    else:
        if kc2 is None:
            raise ValueError("lse_mode 1 needs K^{C2}")
        kc2 = _f32(kc2)
        _load().oracle_block_scores_lse_approx(_p(Q), _p(pos), nr, G, d, _p(kc), nc, p.cmp_len, p.cmp_stride,
                                               _p(kc2), kc2.shape[0], 4 * p.cmp_len, 4 * p.cmp_stride,
                                               float(p.softmax_scale), _p(out), out.shape[1])
    return out[:, :nc]


def topk_blocks(shared: np.ndarray, pos: np.ndarray, p: Params, return_cmp: bool = False):
    """Eq. 6 and Eq. 2.  S^shared [rows, nc] -> I(t) as [rows, topk_total] int32, ascending, -1 padded."""
    shared, pos = _f32(shared), _i32(pos)
    if shared.ndim != 2:
        raise ValueError("shared must be [rows, nc]")
    nr = shared.shape[0]
    stride = shared.shape[1]
    if stride == 0:
        shared = np.zeros((nr, 1), dtype=np.float32)
        stride = 1
    idx = np.full((nr, p.topk_total), -1, dtype=np.int32)
    cmp = None
    cstride = 0
    if return_cmp:
        cstride = int(pos.max()) // p.block_size + 1 if nr else 1
        cmp = np.zeros((nr, cstride), dtype=np.float32)
    _load().oracle_topk_blocks(_p(shared), stride, _p(pos), nr, p.cmp_len, p.cmp_stride, p.block_size,
                               p.pool_len, p.pool_stride, p.pool_pad, p.n_init, p.n_local, p.topk_total,
                               _p(idx), _p(cmp), cstride)
    return (idx, cmp) if return_cmp else idx


def sparse_attn(Q, pos, K, V, idx, p: Params):
    """Appendix Alg. 2 as a definition.  -> O [rows, G, d], lse [rows, G]."""
    Q, pos, K, V, idx = _f32(Q), _i32(pos), _f32(K), _f32(V), _i32(idx)
    nr, G, d = Q.shape
    O = np.zeros((nr, G, d), dtype=np.float32)
    lse = np.zeros((nr, G), dtype=np.float32)
    _load().oracle_sparse_attn(_p(Q), _p(pos), nr, G, d, _p(K), _p(V), K.shape[0], p.block_size, _p(idx),
                               idx.shape[1], float(p.softmax_scale), _p(O), _p(lse))
    return O, lse


def dense_attn(Q, pos, K, V, p: Params):
    """Eq. 1 with a causal mask.  -> O [rows, G, d], lse [rows, G]."""
    Q, pos, K, V = _f32(Q), _i32(pos), _f32(K), _f32(V)
    nr, G, d = Q.shape
    O = np.zeros((nr, G, d), dtype=np.float32)
    lse = np.zeros((nr, G), dtype=np.float32)
    _load().oracle_dense_attn(_p(Q), _p(pos), nr, G, d, _p(K), _p(V), K.shape[0], float(p.softmax_scale),
                              _p(O), _p(lse))
    return O, lse


def attn_bwd(Q, pos, K, V, idx, dO, p: Params):
    """Gradients of stage 4 for a fixed selection (idx None: dense causal attention, Eq. 1) from the definition
    of softmax attention, in float64.  Q, dO [rows, G, d]; K, V [n, d] -> dQ [rows, G, d], dK, dV [n, d]."""
    Q, pos, K, V, dO = _f32(Q), _i32(pos), _f32(K), _f32(V), _f32(dO)
    nr, G, d = Q.shape
    n = K.shape[0]
    dQ = np.zeros((nr, G, d), dtype=np.float64)
    dK = np.zeros((n, d), dtype=np.float64)
    dV = np.zeros((n, d), dtype=np.float64)
    if idx is not None:
        idx = _i32(idx)
    _load().oracle_attn_bwd(_p(Q), _p(pos), nr, G, d, _p(K), _p(V), n, p.block_size, _p(idx),
                            idx.shape[1] if idx is not None else 0, float(p.softmax_scale), _p(dO), _p(dQ), _p(dK),
                            _p(dV))
    return dQ, dK, dV


# --------------------------------------------------------------------------- compositions
def select_blocks(Qh, pos, Kh, p: Params, return_scores: bool = False):
    """Stages 1-3 for one KV head of one sequence: Q rows [rows, G, d], K [n, d] -> idx."""
    kc = compress_k(Kh, p)
    sh = block_scores(Qh, pos, kc, p, kc2=compress_k(Kh, p, level=2) if p.lse_mode == 1 else None)
    idx = topk_blocks(sh, pos, p)
    return (idx, sh, kc) if return_scores else idx


def prefill(q, k, v, cu_seqlens, p: Params, rows: Optional[Sequence[int]] = None, force: Optional[str] = None):
    """The whole switchable path on packed sequences.

    q [T, hq, d]; k, v [hkv, T, d]; cu_seqlens [batch+1].  rows: packed token indices to
    evaluate (default all).  force: None = switch on length, "sparse" / "dense" = ignore it.
    Returns dict(rows, out [R, hq, d], lse [R, hq], idx [hkv, R, topk_total] (-1 rows for dense)).
    """
    q, k, v = _f32(q), _f32(k), _f32(v)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    T, hq, d = q.shape
    hkv = k.shape[0]
    G = hq // hkv
    rows = np.arange(T, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    R = len(rows)
    out = np.zeros((R, hq, d), dtype=np.float32)
    lse = np.zeros((R, hq), dtype=np.float32)
    idx = np.full((hkv, R, p.topk_total), -1, dtype=np.int32)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        sel = np.nonzero((rows >= a) & (rows < b))[0]
        if len(sel) == 0:
            continue
        pos = (rows[sel] - a).astype(np.int32)
        n = b - a
        dense = (n < p.dense_threshold) if force is None else (force == "dense")
        for h in range(hkv):
            Qh = q[rows[sel], h * G:(h + 1) * G, :]
            Kh, Vh = k[h, a:b], v[h, a:b]
            if dense:
                O, L = dense_attn(Qh, pos, Kh, Vh, p)
            else:
                ih = select_blocks(Qh, pos, Kh, p)
                idx[h, sel] = ih
                O, L = sparse_attn(Qh, pos, Kh, Vh, ih, p)
            out[sel, h * G:(h + 1) * G, :] = O
            lse[sel, h * G:(h + 1) * G] = L
    return dict(rows=rows, out=out, lse=lse, idx=idx)


def decode(q, k_cache, v_cache, ctx_lens, p: Params):
    """One decode step per sequence = the row t = L-1 of the sparse path over caches of length L.

    q [batch, hq, d]; k_cache, v_cache [batch, hkv, Lmax, d]; ctx_lens [batch].
    Returns dict(out [batch, hq, d], lse [batch, hq], idx [batch, hkv, topk_total]).
    Sequences shorter than the dense threshold take the dense row instead (idx = -1).
    """
    q, k_cache, v_cache = _f32(q), _f32(k_cache), _f32(v_cache)
    nb, hq, d = q.shape
    hkv = k_cache.shape[1]
    G = hq // hkv
    out = np.zeros((nb, hq, d), dtype=np.float32)
    lse = np.zeros((nb, hq), dtype=np.float32)
    idx = np.full((nb, hkv, p.topk_total), -1, dtype=np.int32)
    for b in range(nb):
        L = int(ctx_lens[b])
        pos = np.array([L - 1], dtype=np.int32)
        for h in range(hkv):
            Qh = q[b:b + 1, h * G:(h + 1) * G, :]
            Kh, Vh = k_cache[b, h, :L], v_cache[b, h, :L]
            if L < p.dense_threshold:
                O, Ls = dense_attn(Qh, pos, Kh, Vh, p)
            else:
                ih = select_blocks(Qh, pos, Kh, p)
                idx[b, h] = ih[0]
                O, Ls = sparse_attn(Qh, pos, Kh, Vh, ih, p)
            out[b, h * G:(h + 1) * G] = O[0]
            lse[b, h * G:(h + 1) * G] = Ls[0]
    return dict(out=out, lse=lse, idx=idx)
