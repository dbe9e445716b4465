"""ctypes binding of libinfllmv2.so: argument marshalling only, one function per C entry point."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libinfllmv2.so")

FP32, BF16 = 0, 1


class InfllmV2Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class Params(ctypes.Structure):
    """Mirror of `infllmv2_params` (paper notation: Sec. 3.2, 3.3, 4.1)."""

    _fields_ = [
        ("dtype", ctypes.c_int32), ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32), ("cmp_len", ctypes.c_int32),
        ("cmp_stride", ctypes.c_int32), ("pool_len", ctypes.c_int32), ("pool_stride", ctypes.c_int32),
        ("pool_pad", ctypes.c_int32), ("n_init", ctypes.c_int32), ("n_local", ctypes.c_int32),
        ("topk_total", ctypes.c_int32), ("dense_threshold", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
        ("lse_mode", ctypes.c_int32),
    ]

    @staticmethod
    def make(dtype: str, num_q_heads: int, num_kv_heads: int, head_dim: int, *, block_size=64, cmp_len=32,
             cmp_stride=16, pool_len=5, pool_stride=4, pool_pad=0, n_init=1, n_local=8, topk_total=64,
             dense_threshold=0, softmax_scale: Optional[float] = None, lse_mode=0) -> "Params":
        scale = float(head_dim) ** -0.5 if softmax_scale is None else float(softmax_scale)
        return Params({"fp32": FP32, "bf16": BF16}[dtype], num_q_heads, num_kv_heads, head_dim, block_size, cmp_len,
                      cmp_stride, pool_len, pool_stride, pool_pad, n_init, n_local, topk_total, dense_threshold,
                      scale, lse_mode)

    @staticmethod
    def from_config(cfg, **over) -> "Params":
        kw = dict(block_size=cfg.block_size, cmp_len=cfg.cmp_len, cmp_stride=cfg.cmp_stride,
                  pool_len=cfg.pool_len, pool_stride=cfg.pool_stride, pool_pad=cfg.pool_pad, n_init=cfg.n_init,
                  n_local=cfg.n_local, topk_total=cfg.topk_total, dense_threshold=cfg.dense_threshold,
                  softmax_scale=cfg.softmax_scale)
        kw.update(over)
        return Params.make(cfg.dtype, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim, **kw)

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == BF16 else torch.float32


_lib = None
_P = ctypes.c_void_p
_I32, _I64, _SZ = ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
_PP = ctypes.POINTER(Params)

_SIGNATURES = {
    "infllmv2_num_cmp": (_I32, [_PP, _I32]),
    "infllmv2_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "infllmv2_version": (ctypes.c_char_p, []),
    "infllmv2_compress_k": (ctypes.c_int, [_PP, _P, _I64, _I64, _P, _P, _I32, _P, _P, _I64, _P]),
    "infllmv2_compress_k_append": (ctypes.c_int, [_PP, _P, _I64, _I64, _I64, _P, _I64, _P, _P, _P, _P, _I32, _P]),
    "infllmv2_workspace_bytes": (_SZ, [ctypes.c_int, _PP, _I32, _I64, _I32]),
    "infllmv2_block_scores": (ctypes.c_int, [_PP, _P, _P, _I64, _P, _P, _P, _I32, _P, _I64, _P, _SZ, _P]),
    "infllmv2_topk_blocks": (ctypes.c_int, [_PP, _P, _I64, _P, _P, _I32, _P, _P]),
    "infllmv2_block_scores_pooled": (ctypes.c_int, [_PP, _P, _P, _I64, _P, _P, _P, _I32, _P, _I64, _P, _SZ, _P]),
    "infllmv2_topk_pooled": (ctypes.c_int, [_PP, _P, _I64, _P, _P, _I32, _P, _P]),
    "infllmv2_sparse_attn_fwd": (ctypes.c_int, [_PP, _P, _P, _P, _I64, _I64, _P, _P, _P, _I32, _P, _P, _P, _SZ, _P]),
    "infllmv2_dense_attn_fwd": (ctypes.c_int, [_PP, _P, _P, _P, _I64, _I64, _P, _P, _I32, _P, _P, _P, _SZ, _P]),
    "infllmv2_sparse_attn_bwd": (ctypes.c_int, [_PP, _P, _P, _P, _I64, _I64, _P, _P, _P, _P, _P, _P, _I32, _P, _P, _P,
                                                _P, _SZ, _P]),
    "infllmv2_sparse_decode": (ctypes.c_int, [_PP, _P, _P, _P, _I64, _I64, _I64, _P, _I64, _P, _P, _I32, _P, _P, _P,
                                              _P, _SZ, _P]),
    "infllmv2_decode_workspace_bytes": (_SZ, [_PP, _I32, _I32]),
    "infllmv2_sparse_decode_static": (ctypes.c_int, [_PP, _P, _P, _P, _I64, _I64, _I64, _P, _I64, _P, _P, _I32, _P, _P, _P,
                                                     _P]),
    "infllmv2_sparse_decode_static_capacity": (_SZ, []),
}


def lib() -> ctypes.CDLL:
    """Load libinfllmv2.so (no fallback: a missing library is an error)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "(or python paper_2509_24663_amd/build.py) first; there is no CPU fallback")
        L = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def exported_symbols() -> Sequence[str]:
    return tuple(_SIGNATURES)


def status_string(status: int) -> str:
    return lib().infllmv2_status_string(int(status)).decode()


def version() -> str:
    return lib().infllmv2_version().decode()


def num_cmp(p: Params, n: int) -> int:
    return int(lib().infllmv2_num_cmp(ctypes.byref(p), int(n)))


def _check(st: int, where: str):
    if st != 0:
        raise InfllmV2Error(st, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


# `op` of infllmv2_workspace_bytes (enum infllmv2_op)
OP_COMPRESS_K, OP_BLOCK_SCORES, OP_TOPK_BLOCKS, OP_SPARSE_ATTN_FWD, OP_DENSE_ATTN_FWD, OP_SPARSE_DECODE = range(6)
OP_BLOCK_SCORES_POOLED, OP_TOPK_POOLED, OP_SPARSE_ATTN_BWD, OP_SPARSE_ATTN_BWD_MIN, OP_COMPRESS_K_APPEND = range(6, 11)


def workspace_bytes(op: int, p: Params, batch: int, total_tokens: int, max_seqlen: int) -> int:
    """Bytes of scratch call `op` needs at most for such a batch (host helper, no GPU needed)."""
    return int(lib().infllmv2_workspace_bytes(int(op), ctypes.byref(p), int(batch), int(total_tokens), int(max_seqlen)))


def _workspace(op: int, p: Params, cu_h: torch.Tensor, device, given: Optional[torch.Tensor]):
    """The caller's scratch tensor, or a new one of the size the library asks for (None when it asks for none)."""
    if given is not None:
        return given
    batch = cu_h.numel() - 1
    max_len = int((cu_h[1:] - cu_h[:-1]).max()) if batch else 0
    need = workspace_bytes(op, p, batch, int(cu_h[-1]), max_len)
    return torch.empty(need, dtype=torch.uint8, device=device) if need else None


def _ws_args(ws: Optional[torch.Tensor]):
    return (None, 0) if ws is None else (ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size())


class SeqInfo:
    """cu_seqlens as the ABI wants it: a host int32 array plus a device copy, made once and reused."""

    def __init__(self, cu_seqlens):
        self.cu_h = torch.as_tensor(cu_seqlens, dtype=torch.int32, device="cpu").contiguous()
        self.cu_d = self.cu_h.cuda()
        self.batch = self.cu_h.numel() - 1
        lens = (self.cu_h[1:] - self.cu_h[:-1])
        self.lens = lens.tolist()
        self.max_len = int(lens.max()) if self.batch else 0
        self.total = int(self.cu_h[-1])


def _cu_pair(cu_seqlens):
    """host int32 tensor + device copy (pass a SeqInfo to avoid the copy on every call)"""
    si = cu_seqlens if isinstance(cu_seqlens, SeqInfo) else SeqInfo(cu_seqlens)
    return si.cu_h, si.cu_d


def _kv_strides(k: torch.Tensor):
    """k is [hkv, T, d] (head-major) or any view with d contiguous: returns (tok_stride, head_stride)."""
    assert k.dim() == 3 and k.stride(2) == 1
    return k.stride(1), k.stride(0)


# ---------------------------------------------------------------------------------- stage wrappers
def compress_k(p: Params, k: torch.Tensor, cu_seqlens, out=None):
    """Stage 1.  k [hkv, T, d] (device).  Returns kc [hkv, total_c, d] fp32, cu_seqlens_c (device int32).
    out: optional (kc, cu_seqlens_c) buffers to reuse."""
    cu_h, cu_d = _cu_pair(cu_seqlens)
    batch = cu_h.numel() - 1
    if out is None:
        lens = (cu_h[1:] - cu_h[:-1]).tolist()
        total_c = sum(num_cmp(p, n) for n in lens)
        kc = torch.empty((p.num_kv_heads, max(total_c, 1), p.head_dim), dtype=torch.float32, device=k.device)
        cu_c = torch.empty(batch + 1, dtype=torch.int32, device=k.device)
    else:
        kc, cu_c = out
    ts, hs = _kv_strides(k)
    st = lib().infllmv2_compress_k(ctypes.byref(p), _ptr(k), ts, hs, _ptr(cu_h), _ptr(cu_d), batch, _ptr(kc),
                                   _ptr(cu_c), kc.shape[1], _stream())
    _check(st, "infllmv2_compress_k")
    return kc, cu_c


def compress_k_append(p: Params, k_cache: torch.Tensor, kc_cache: torch.Tensor, prev_lens, ctx_lens):
    """Brings a decode compressed-key cache up to date in place.  k_cache [B, hkv, Lmax, d]; kc_cache
    [B, hkv, max_nc, d] fp32; prev_lens / ctx_lens: sequences of ints or DecodeInfo (cache lengths then and now)."""
    pv = prev_lens if isinstance(prev_lens, DecodeInfo) else DecodeInfo(prev_lens)
    cx = ctx_lens if isinstance(ctx_lens, DecodeInfo) else DecodeInfo(ctx_lens)
    assert k_cache.dim() == 4 and k_cache.stride(3) == 1 and kc_cache.dim() == 4 and kc_cache.is_contiguous()
    st = lib().infllmv2_compress_k_append(ctypes.byref(p), _ptr(k_cache), k_cache.stride(0), k_cache.stride(1),
                                          k_cache.stride(2), _ptr(kc_cache), kc_cache.stride(1), _ptr(pv.ctx_h),
                                          _ptr(pv.ctx_d), _ptr(cx.ctx_h), _ptr(cx.ctx_d), cx.batch, _stream())
    _check(st, "infllmv2_compress_k_append")
    return kc_cache


def block_scores(p: Params, q: torch.Tensor, kc: torch.Tensor, cu_seqlens, cu_seqlens_c: torch.Tensor,
                 out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """Stage 2.  q [T, hq, d]; returns S^shared [hkv, T, row_stride] fp32 (entries beyond v(t) unspecified).
    workspace: a uint8 device tensor of workspace_bytes(OP_BLOCK_SCORES, ...) bytes to reuse (else made here)."""
    assert q.is_contiguous() and kc.is_contiguous()
    cu_h, cu_d = _cu_pair(cu_seqlens)
    batch = cu_h.numel() - 1
    max_len = int((cu_h[1:] - cu_h[:-1]).max()) if batch else 0
    rs = max(4, (num_cmp(p, max_len) + 3) // 4 * 4)
    if out is None:
        out = torch.empty((p.num_kv_heads, q.shape[0], rs), dtype=torch.float32, device=q.device)
    ws = _workspace(OP_BLOCK_SCORES, p, cu_h, q.device, workspace)
    st = lib().infllmv2_block_scores(ctypes.byref(p), _ptr(q), _ptr(kc), kc.shape[1], _ptr(cu_h), _ptr(cu_d),
                                     _ptr(cu_seqlens_c), batch, _ptr(out), out.shape[2], *_ws_args(ws), _stream())
    _check(st, "infllmv2_block_scores")
    return out


def topk_blocks(p: Params, s_shared: torch.Tensor, cu_seqlens, out: Optional[torch.Tensor] = None):
    """Stage 3.  s_shared [hkv, T, row_stride] -> block_idx [hkv, T, topk_total] int32."""
    cu_h, cu_d = _cu_pair(cu_seqlens)
    batch = cu_h.numel() - 1
    if out is None:
        out = torch.empty((p.num_kv_heads, s_shared.shape[1], p.topk_total), dtype=torch.int32, device=s_shared.device)
    st = lib().infllmv2_topk_blocks(ctypes.byref(p), _ptr(s_shared), s_shared.shape[2], _ptr(cu_h), _ptr(cu_d), batch,
                                    _ptr(out), _stream())
    _check(st, "infllmv2_topk_blocks")
    return out


def block_scores_pooled(p: Params, q: torch.Tensor, kc: torch.Tensor, cu_seqlens, cu_seqlens_c: torch.Tensor,
                        out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """Stages 2 with the max-pooling fused.  Returns S^cmp [hkv, T, row_stride >= ceil(max len / 64)] fp32; entry j of
    a row is written iff the block's pooling window holds a visible key."""
    cu_h, cu_d = _cu_pair(cu_seqlens)
    batch = cu_h.numel() - 1
    max_len = int((cu_h[1:] - cu_h[:-1]).max()) if batch else 0
    if out is None:
        rs = max(1, (max_len + p.block_size - 1) // p.block_size)
        out = torch.empty((p.num_kv_heads, q.shape[0], rs), dtype=torch.float32, device=q.device)
    assert q.is_contiguous() and kc.is_contiguous()
    ws = _workspace(OP_BLOCK_SCORES_POOLED, p, cu_h, q.device, workspace)
    st = lib().infllmv2_block_scores_pooled(ctypes.byref(p), _ptr(q), _ptr(kc), kc.shape[1], _ptr(cu_h), _ptr(cu_d),
                                            _ptr(cu_seqlens_c), batch, _ptr(out), out.shape[2], *_ws_args(ws),
                                            _stream())
    _check(st, "infllmv2_block_scores_pooled")
    return out


def topk_pooled(p: Params, s_cmp: torch.Tensor, cu_seqlens, out: Optional[torch.Tensor] = None):
    """Stage 3 on pooled scores.  s_cmp [hkv, T, row_stride] -> block_idx [hkv, T, topk_total] int32."""
    cu_h, cu_d = _cu_pair(cu_seqlens)
    batch = cu_h.numel() - 1
    if out is None:
        out = torch.empty((p.num_kv_heads, s_cmp.shape[1], p.topk_total), dtype=torch.int32, device=s_cmp.device)
    st = lib().infllmv2_topk_pooled(ctypes.byref(p), _ptr(s_cmp), s_cmp.shape[2], _ptr(cu_h), _ptr(cu_d), batch,
                                    _ptr(out), _stream())
    _check(st, "infllmv2_topk_pooled")
    return out


def sparse_attn_fwd(p: Params, q, k, v, block_idx, cu_seqlens, out=None, lse=None, workspace=None):
    """Stage 4.  Returns (out [T, hq, d], lse [hq, T]).  workspace: scratch tensor to reuse (else made here)."""
    cu_h, cu_d = _cu_pair(cu_seqlens)
    batch = cu_h.numel() - 1
    out = torch.empty_like(q) if out is None else out
    lse = torch.empty((p.num_q_heads, q.shape[0]), dtype=torch.float32, device=q.device) if lse is None else lse
    ts, hs = _kv_strides(k)
    assert _kv_strides(v) == (ts, hs)
    assert q.is_contiguous() and out.is_contiguous() and lse.is_contiguous() and block_idx.is_contiguous()
    ws = _workspace(OP_SPARSE_ATTN_FWD, p, cu_h, q.device, workspace)
    st = lib().infllmv2_sparse_attn_fwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), ts, hs, _ptr(block_idx),
                                        _ptr(cu_h), _ptr(cu_d), batch, _ptr(out), _ptr(lse), *_ws_args(ws), _stream())
    _check(st, "infllmv2_sparse_attn_fwd")
    return out, lse


def dense_attn_fwd(p: Params, q, k, v, cu_seqlens, out=None, lse=None, workspace=None):
    """Dense causal GQA attention.  Returns (out [T, hq, d], lse [hq, T])."""
    cu_h, cu_d = _cu_pair(cu_seqlens)
    batch = cu_h.numel() - 1
    out = torch.empty_like(q) if out is None else out
    lse = torch.empty((p.num_q_heads, q.shape[0]), dtype=torch.float32, device=q.device) if lse is None else lse
    ts, hs = _kv_strides(k)
    assert _kv_strides(v) == (ts, hs)
    assert q.is_contiguous() and out.is_contiguous() and lse.is_contiguous()
    ws = _workspace(OP_DENSE_ATTN_FWD, p, cu_h, q.device, workspace)
    st = lib().infllmv2_dense_attn_fwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), ts, hs, _ptr(cu_h), _ptr(cu_d),
                                       batch, _ptr(out), _ptr(lse), *_ws_args(ws), _stream())
    _check(st, "infllmv2_dense_attn_fwd")
    return out, lse


def sparse_attn_bwd(p: Params, q, k, v, block_idx, out, lse, dout, cu_seqlens, dq=None, dk=None, dv=None,
                    workspace=None, sel_bitmap_max_bytes: int = 512 << 20):
    """Gradients of stage 4 for a given selection (block_idx None: dense).  Returns (dq like q, dk, dv float32
    [hkv, T, d]).  workspace: scratch tensor to reuse; when it is made here it includes room for the selection
    bitmap unless that would take more than sel_bitmap_max_bytes (0: never)."""
    cu_h, cu_d = _cu_pair(cu_seqlens)
    batch = cu_h.numel() - 1
    ts, hs = _kv_strides(k)
    assert _kv_strides(v) == (ts, hs)
    T = q.shape[0]
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty((p.num_kv_heads, T, p.head_dim), dtype=torch.float32, device=q.device) if dk is None else dk
    dv = torch.empty((p.num_kv_heads, T, p.head_dim), dtype=torch.float32, device=q.device) if dv is None else dv
    assert dout.is_contiguous() and out.is_contiguous() and dq.is_contiguous() and dk.is_contiguous() and dv.is_contiguous()
    assert q.is_contiguous() and lse.is_contiguous()
    if workspace is None:
        max_len = int((cu_h[1:] - cu_h[:-1]).max()) if batch else 0
        full = workspace_bytes(OP_SPARSE_ATTN_BWD, p, batch, T, max_len)
        least = workspace_bytes(OP_SPARSE_ATTN_BWD_MIN, p, batch, T, max_len)
        need = full if block_idx is not None and full - least <= sel_bitmap_max_bytes else least
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device) if need else None
    st = lib().infllmv2_sparse_attn_bwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), ts, hs, _ptr(block_idx), _ptr(out),
                                        _ptr(lse), _ptr(dout), _ptr(cu_h), _ptr(cu_d), batch, _ptr(dq), _ptr(dk),
                                        _ptr(dv), *_ws_args(workspace), _stream())
    _check(st, "infllmv2_sparse_attn_bwd")
    return dq, dk, dv


def decode_workspace_bytes(p: Params, batch: int, max_ctx_len: int) -> int:
    return int(lib().infllmv2_decode_workspace_bytes(ctypes.byref(p), int(batch), int(max_ctx_len)))


class DecodeInfo:
    """ctx_lens as the ABI wants them (host + device copy), made once per step and reusable."""

    def __init__(self, ctx_lens):
        self.ctx_h = torch.as_tensor(ctx_lens, dtype=torch.int32, device="cpu").contiguous()
        self.ctx_d = self.ctx_h.cuda()
        self.batch = self.ctx_h.numel()
        self.max_ctx = int(self.ctx_h.max()) if self.batch else 0


def sparse_decode(p: Params, q, k_cache, v_cache, kc_cache, ctx_lens, workspace=None, return_idx=True, out=None,
                  lse=None, idx=None):
    """Decode step.  q [B, hq, d]; k_cache/v_cache [B, hkv, Lmax, d]; kc_cache [B, hkv, max_nc, d] fp32.
    ctx_lens: a sequence of ints or a DecodeInfo.  out / lse / idx / workspace: optional buffers to reuse.
    Returns (out [B, hq, d], lse [B, hq], block_idx [B, hkv, topk_total] or None)."""
    di = ctx_lens if isinstance(ctx_lens, DecodeInfo) else DecodeInfo(ctx_lens)
    B = q.shape[0]
    if workspace is None:
        workspace = torch.empty(max(decode_workspace_bytes(p, B, di.max_ctx), 256), dtype=torch.uint8, device=q.device)
    out = torch.empty_like(q) if out is None else out
    lse = torch.empty((B, p.num_q_heads), dtype=torch.float32, device=q.device) if lse is None else lse
    if idx is None and return_idx:
        idx = torch.empty((B, p.num_kv_heads, p.topk_total), dtype=torch.int32, device=q.device)
    assert k_cache.dim() == 4 and k_cache.stride(3) == 1 and k_cache.stride() == v_cache.stride()
    assert kc_cache.dim() == 4 and kc_cache.is_contiguous()
    st = lib().infllmv2_sparse_decode(ctypes.byref(p), _ptr(q), _ptr(k_cache), _ptr(v_cache), k_cache.stride(0),
                                      k_cache.stride(1), k_cache.stride(2), _ptr(kc_cache), kc_cache.stride(1),
                                      _ptr(di.ctx_h), _ptr(di.ctx_d), B, _ptr(idx), _ptr(out), _ptr(lse),
                                      _ptr(workspace), workspace.numel(), _stream())
    _check(st, "infllmv2_sparse_decode")
    return out, lse, idx


def sparse_decode_static_capacity() -> int:
    return int(lib().infllmv2_sparse_decode_static_capacity())


def sparse_decode_static(p: Params, q, k_cache, v_cache, kc_cache, ctx_lens, out, lse, idx=None):
    """Decode step through the entry point that allocates nothing: scratch is a fixed array inside the library, and
    every output buffer is the caller's (out [B, hq, d], lse [B, hq], idx [B, hkv, topk_total] or None)."""
    di = ctx_lens if isinstance(ctx_lens, DecodeInfo) else DecodeInfo(ctx_lens)
    assert k_cache.dim() == 4 and k_cache.stride(3) == 1 and k_cache.stride() == v_cache.stride()
    assert kc_cache.dim() == 4 and kc_cache.is_contiguous() and q.is_contiguous() and out.is_contiguous()
    st = lib().infllmv2_sparse_decode_static(ctypes.byref(p), _ptr(q), _ptr(k_cache), _ptr(v_cache), k_cache.stride(0),
                                             k_cache.stride(1), k_cache.stride(2), _ptr(kc_cache), kc_cache.stride(1),
                                             _ptr(di.ctx_h), _ptr(di.ctx_d), q.shape[0], _ptr(idx), _ptr(out), _ptr(lse),
                                             _stream())
    _check(st, "infllmv2_sparse_decode_static")
    return out, lse, idx


def sparse_prefill(p: Params, q, k, v, cu_seqlens, buffers: Optional[dict] = None, fused_pool: bool = False):
    """The four stages back to back (a convenience for tests and the benchmark; no arithmetic here).
    buffers: a dict returned by an earlier call, whose tensors are then reused (nothing is allocated).
    fused_pool: stages 2 and 3 through the pooled entry points (s_cmp instead of s_shared in the result).
    Returns dict(out, lse, block_idx, s_shared | s_cmp, kc, cu_seqlens_c)."""
    b = buffers or {}
    si = cu_seqlens if isinstance(cu_seqlens, SeqInfo) else SeqInfo(cu_seqlens)
    kc, cu_c = compress_k(p, k, si, out=(b["kc"], b["cu_seqlens_c"]) if b else None)
    ws_scores = b.get("ws_scores")
    if ws_scores is None:
        ws_scores = _workspace(OP_BLOCK_SCORES_POOLED if fused_pool else OP_BLOCK_SCORES, p, si.cu_h, q.device, None)
    if fused_pool:
        sc = block_scores_pooled(p, q, kc, si, cu_c, out=b.get("s_cmp"), workspace=ws_scores)
        idx = topk_pooled(p, sc, si, out=b.get("block_idx"))
        scores = dict(s_cmp=sc)
    else:
        sh = block_scores(p, q, kc, si, cu_c, out=b.get("s_shared"), workspace=ws_scores)
        idx = topk_blocks(p, sh, si, out=b.get("block_idx"))
        scores = dict(s_shared=sh)
    ws_attn = b.get("ws_attn")
    if ws_attn is None:
        ws_attn = _workspace(OP_SPARSE_ATTN_FWD, p, si.cu_h, q.device, None)
    out, lse = sparse_attn_fwd(p, q, k, v, idx, si, out=b.get("out"), lse=b.get("lse"), workspace=ws_attn)
    return dict(out=out, lse=lse, block_idx=idx, kc=kc, cu_seqlens_c=cu_c, ws_attn=ws_attn, ws_scores=ws_scores,
                **scores)
