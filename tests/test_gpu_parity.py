"""GPU parity: every stage of the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integer results (block lists given identical scores) must match bit for bit; end-to-end
selections may differ only at near-ties (1e-3 relative); attention outputs must be within max-abs 1e-4
(fp32) or max-abs 2e-2 / mean-abs 2e-3 (bf16) -- also when the oracle is fed the GPU's own selection,
which separates attention error from selection error."""
import numpy as np
import pytest
import torch

import synth
from helpers import (SCORE_RTOL, TIE_FLIP_RATE_MAX, assert_out_close, check_selection, prefill_lse_atol, to_dev,
                     to_np)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def m():
    import paper_2509_24663_amd as m
    m.lib()
    assert torch.cuda.is_available()
    return m


def _params(m, oracle, dtype, hq, hkv, d, **kw):
    gp = m.Params.make(dtype, hq, hkv, d, **kw)
    op = oracle.Params(block_size=gp.block_size, cmp_len=gp.cmp_len, cmp_stride=gp.cmp_stride, pool_len=gp.pool_len,
                       pool_stride=gp.pool_stride, pool_pad=gp.pool_pad, n_init=gp.n_init, n_local=gp.n_local,
                       topk_total=gp.topk_total, dense_threshold=gp.dense_threshold,
                       softmax_scale=float(gp.softmax_scale), lse_mode=gp.lse_mode)
    return gp, op


def _run_prefill_case(m, oracle, w, gp, op, dtype, rows=None, check_stages=True, fused_pool=False):
    """Full sparse path on one packed workload, checked on `rows` (packed token indices, default all).
    fused_pool: stages 2-3 through the pooled entry points (their scores are then compared per selection block).
    Returns statistics: rows whose list differs from the oracle's by near-ties, the largest relative score error
    seen, the largest output / lse errors; the tie-flip rate is bounded here, so a loss of precision in stage 2
    cannot hide behind the tie rule."""
    cu = w["cu_seqlens"]
    T, hq, d = w["q"].shape
    hkv = w["k"].shape[0]
    G = hq // hkv
    q, k, v = (to_dev(w[x], dtype) for x in ("q", "k", "v"))
    res = m.sparse_prefill(gp, q, k, v, cu, fused_pool=fused_pool)
    torch.cuda.synchronize()
    rows = np.arange(T) if rows is None else np.unique(np.asarray(rows))
    rows_d = torch.from_numpy(rows).cuda()
    # only the sampled rows leave the GPU (S^shared alone is 8.6 GB at 128K)
    out_g = to_np(res["out"][rows_d])                       # [R, hq, d]
    lse_g = to_np(res["lse"][:, rows_d])                    # [hq, R]
    idx_g = to_np(res["block_idx"][:, rows_d])              # [hkv, R, K]
    sc_g = to_np(res["s_cmp" if fused_pool else "s_shared"][:, rows_d])     # [hkv, R, rs]
    kc_g = to_np(res["kc"])
    stats = dict(rows_diff=0, blocks_diff=0, rows=0, max_abs=0.0, score_rel=0.0, lse_abs=0.0)
    cu_c = to_np(res["cu_seqlens_c"].int())
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        n = b - a
        loc = np.nonzero((rows >= a) & (rows < b))[0]        # positions in the sampled arrays
        if len(loc) == 0:
            continue
        sel = rows[loc]
        pos = (sel - a).astype(np.int32)
        dense = n < op.dense_threshold
        for h in range(hkv):
            Qh = w["q"][sel, h * G:(h + 1) * G]
            Kh, Vh = w["k"][h, a:b], w["v"][h, a:b]
            if dense:
                O, L = oracle.dense_attn(Qh, pos, Kh, Vh, op)
                assert np.all(idx_g[h, loc] == -1)
                assert_out_close(out_g[loc, h * G:(h + 1) * G], O, dtype, "out end-to-end (dense sequence)")
                continue
            kc_o = oracle.compress_k(Kh, op)
            nc = kc_o.shape[0]
            assert cu_c[s + 1] - cu_c[s] == nc
            if check_stages:
                np.testing.assert_allclose(kc_g[h, cu_c[s]:cu_c[s] + nc], kc_o, rtol=0,
                                           atol=2e-6 * max(1.0, float(np.abs(kc_o).max()) if nc else 1.0))
            sh_o = oracle.block_scores(Qh, pos, kc_o, op,
                                       kc2=oracle.compress_k(Kh, op, level=2) if op.lse_mode else None)
            idx_o, cmp_o = oracle.topk_blocks(sh_o, pos, op, return_cmp=True)
            if check_stages:
                # stage 2 rounds K^{C1} to an 11-bit significand (fp16 MFMA operands): per-logit error ~1e-4, so
                # scores agree to a few 1e-4 relative -- inside the 1e-3 tie window; the largest error is reported
                shg_rows = np.zeros_like(sh_o)
                for r, t in enumerate(pos):
                    if fused_pool:
                        # entry j is defined iff block j's (clipped) pooling window holds a visible key
                        vis = oracle.visible_cmp(int(t), op)
                        js = [j for j in range(int(t) // op.block_size + 1)
                              if max(op.pool_stride * j - op.pool_pad, 0) < vis]
                        got, want = sc_g[h, loc[r], js], cmp_o[r, js]
                    else:
                        vis = oracle.visible_cmp(int(t), op)
                        got, want = sc_g[h, loc[r], :vis], sh_o[r, :vis]
                        shg_rows[r, :vis] = got
                    if len(want):
                        # |got - want| <= 1e-7 + SCORE_RTOL |want|, reported as the relative part
                        err = np.maximum(np.abs(got - want) - 1e-7, 0.0) / np.maximum(np.abs(want), 1e-30)
                        stats["score_rel"] = max(stats["score_rel"], float(err.max()))
                assert stats["score_rel"] <= SCORE_RTOL, f"stage-2 scores off by {stats['score_rel']:.3e} relative"
                if not fused_pool:
                    # stage 3 alone: oracle top-k of the GPU's scores must equal the GPU's list bit for bit
                    np.testing.assert_array_equal(idx_g[h, loc], oracle.topk_blocks(shg_rows, pos, op))
            rd, bd = check_selection(idx_g[h, loc], idx_o, cmp_o, pos, op.n_init, op.n_local)
            stats["rows_diff"] += rd
            stats["blocks_diff"] += bd
            stats["rows"] += len(loc)
            # attention error alone: oracle attention over the GPU's selection
            O_iso, L_iso = oracle.sparse_attn(Qh, pos, Kh, Vh, idx_g[h, loc], op)
            mx, _ = assert_out_close(out_g[loc, h * G:(h + 1) * G], O_iso, dtype, "out | GPU selection")
            stats["max_abs"] = max(stats["max_abs"], mx)
            lerr = float(np.abs(lse_g[h * G:(h + 1) * G, loc].T - L_iso).max())
            stats["lse_abs"] = max(stats["lse_abs"], lerr)
            assert lerr <= prefill_lse_atol(dtype), f"lse off by {lerr:.3e}"
            # end to end: every row whose list equals the oracle's must also match the oracle's output (rows whose
            # lists differ by a near-tie legitimately attend to another block)
            same = (idx_g[h, loc] == idx_o).all(axis=1)
            if same.any():
                assert_out_close(out_g[loc[same], h * G:(h + 1) * G], O_iso[same], dtype, "out end-to-end")
    assert stats["rows_diff"] <= TIE_FLIP_RATE_MAX * max(stats["rows"], 1) + 1, (
        f"{stats['rows_diff']} of {stats['rows']} sampled rows differ from the oracle's lists by near-ties")
    return stats


# ----------------------------------------------------------------------------------------------- configs
def test_c1_tiny_fp32_full(m, oracle):
    """Workload C1 of synth.CONFIGS in full: fp32, n 2048, 4 q heads / 1 kv head, d 64, top-k 8 (1 init + 2 local)."""
    cfg = synth.CONFIGS["C1"]
    w = synth.make_config(cfg)
    gp, op = m.Params.from_config(cfg), oracle.Params.from_config(cfg)
    st = _run_prefill_case(m, oracle, w, gp, op, "fp32")
    assert st["rows_diff"] == 0, st


@pytest.mark.parametrize("n", [1, 31, 32, 63, 64, 65, 200, 1000, 1537])
def test_ragged_lengths_fp32(m, oracle, n):
    w = synth.make_prefill(n, 4, 2, 64, seed=100 + n, dtype="fp32")
    gp, op = _params(m, oracle, "fp32", 4, 2, 64, n_init=1, n_local=2, topk_total=6)
    _run_prefill_case(m, oracle, w, gp, op, "fp32")


@pytest.mark.parametrize("shape", [(8, 2, 128), (3, 3, 64), (16, 1, 64), (6, 2, 128)])
def test_head_shapes_bf16_generic(m, oracle, shape):
    hq, hkv, d = shape
    w = synth.make_prefill(700, hq, hkv, d, seed=7, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", hq, hkv, d, n_init=1, n_local=2, topk_total=5)
    _run_prefill_case(m, oracle, w, gp, op, "bf16")


@pytest.mark.parametrize("n", [257, 2048, 4500])
def test_paper_head_shape_bf16(m, oracle, n):
    """h_q 32 / h_kv 2 / d 128 (the paper's model shape): the MFMA kernels' home."""
    w = synth.make_prefill(n, 32, 2, 128, seed=300 + n, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=8, topk_total=16)
    _run_prefill_case(m, oracle, w, gp, op, "bf16")


@pytest.mark.parametrize("qexp,kexp", [(14, -7), (-3, 17), (0, 0)])
def test_scores_survive_large_magnitudes(m, oracle, qexp, kexp):
    """Stage 2 works on fp16 operands internally; power-of-two input scalings that leave every logit unchanged
    (compensated in softmax_scale) must leave the selection unchanged, including magnitudes beyond 65504."""
    n = 3000
    w = synth.make_prefill(n, 32, 2, 128, seed=404, dtype="bf16")
    w["q"] = (w["q"] * np.float32(2.0 ** qexp)).astype(np.float32)       # exact in bf16: power-of-two scaling
    w["k"] = (w["k"] * np.float32(2.0 ** kexp)).astype(np.float32)
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=4, topk_total=12,
                     softmax_scale=128 ** -0.5 * 2.0 ** (-qexp - kexp))
    _run_prefill_case(m, oracle, w, gp, op, "bf16")


@pytest.mark.parametrize("shape", [("bf16", 32, 2, 128, 2300), ("bf16", 32, 2, 128, 200), ("fp32", 4, 1, 64, 1500),
                                   ("bf16", 8, 2, 64, 700)])
def test_lse_approximation_prefill(m, oracle, shape):
    """Stage 2 with the LSE Approximation (Sec. 3.4, Eq. 7; lse_mode 1) against the oracle's variant, through the
    whole path: MFMA kernel (bf16, G 16, d 128) and generic kernel (other shapes); rows below token 127 see no
    coarse key and must get all-zero scores."""
    dtype, hq, hkv, d, n = shape
    w = synth.make_prefill(n, hq, hkv, d, seed=77, dtype=dtype)
    gp, op = _params(m, oracle, dtype, hq, hkv, d, n_init=1, n_local=2, topk_total=10, lse_mode=1)
    assert op.lse_mode == 1
    _run_prefill_case(m, oracle, w, gp, op, dtype)
    res = m.sparse_prefill(gp, *(to_dev(w[x], dtype) for x in ("q", "k", "v")), w["cu_seqlens"])
    sh = to_np(res["s_shared"])
    for t in range(31, min(n, 127)):
        assert np.all(sh[:, t, :oracle.visible_cmp(t, op)] == 0)


def test_lse_approximation_varlen_and_decode(m, oracle):
    """lse_mode 1 on packed sequences of different lengths (each has its own coarse-key count), and in the decode
    entry point, which must give the last prefill row."""
    lengths = (90, 128, 191, 1000, 2049)
    w = synth.make_varlen(lengths, 32, 2, 128, seed=5, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=3, topk_total=9, lse_mode=1)
    _run_prefill_case(m, oracle, w, gp, op, "bf16")
    ctx = [300, 1500, 127, 64, 6100]
    dw = synth.make_decode(ctx, 32, 2, 128, seed=6, dtype="bf16")
    _check_decode(m, oracle, dw, ctx, gp, op, "bf16")


@pytest.mark.parametrize("cfg", [(1, 1, 4), (2, 3, 9), (0, 1, 3), (1, 8, 64)])
@pytest.mark.parametrize("pad", [0, 1])
def test_topk_stage_bit_exact_on_tied_scores(m, oracle, cfg, pad):
    """Stage 3 alone on scores with many exact ties: the block lists must equal the oracle's bit for bit."""
    n_init, n_local, total = cfg
    n = 6000
    gp, op = _params(m, oracle, "fp32", 4, 2, 64, n_init=n_init, n_local=n_local, topk_total=total, pool_pad=pad)
    nc = oracle.num_cmp(n, op)
    rs = (nc + 3) // 4 * 4
    rng = np.random.default_rng(5)
    sh = np.zeros((2, n, rs), np.float32)
    for t in range(n):
        v = oracle.visible_cmp(t, op)
        sh[:, t, :v] = rng.integers(0, 40, (2, v)).astype(np.float32) / 16
        sh[:, t, v:] = 77.0          # garbage beyond the visible prefix must be ignored
    idx = to_np(m.topk_blocks(gp, torch.from_numpy(sh).cuda(), [0, n]))
    pos = np.arange(n, dtype=np.int32)
    for h in range(2):
        clean = sh[h].copy()
        for t in range(n):
            clean[t, oracle.visible_cmp(t, op):] = 0
        np.testing.assert_array_equal(idx[h], oracle.topk_blocks(clean[:, :nc], pos, op))


def test_dense_attention(m, oracle):
    for dtype, hq, hkv, d, n in [("fp32", 4, 1, 64, 777), ("bf16", 32, 2, 128, 1100), ("bf16", 8, 2, 64, 300)]:
        w = synth.make_prefill(n, hq, hkv, d, seed=9, dtype=dtype)
        gp, op = _params(m, oracle, dtype, hq, hkv, d)
        q, k, v = (to_dev(w[x], dtype) for x in ("q", "k", "v"))
        out, lse = m.dense_attn_fwd(gp, q, k, v, [0, n])
        torch.cuda.synchronize()
        ref = oracle.prefill(w["q"], w["k"], w["v"], [0, n], op, force="dense")
        assert_out_close(to_np(out), ref["out"], dtype, "dense out")
        np.testing.assert_allclose(to_np(lse).T, ref["lse"], atol=prefill_lse_atol(dtype))


def test_sparse_equals_dense_when_all_blocks_kept(m, oracle):
    """Invariant: with top-k covering every block the sparse path is dense causal attention."""
    n = 1000
    w = synth.make_prefill(n, 32, 2, 128, seed=12, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=8, topk_total=16)
    q, k, v = (to_dev(w[x], "bf16") for x in ("q", "k", "v"))
    res = m.sparse_prefill(gp, q, k, v, [0, n])
    dn, dl = m.dense_attn_fwd(gp, q, k, v, [0, n])
    torch.cuda.synchronize()
    assert_out_close(to_np(res["out"]), to_np(dn), "bf16")
    np.testing.assert_allclose(to_np(res["lse"]), to_np(dl), atol=2e-3)


def test_varlen_switch(m, oracle):
    """Packed sequences on both sides of the dense/sparse threshold (the shape of workload C5, smaller)."""
    lens = [100, 1024, 64, 2500, 1023, 1]
    w = synth.make_varlen(lens, 32, 2, 128, seed=77, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=4, topk_total=10, dense_threshold=1024)
    st = _run_prefill_case(m, oracle, w, gp, op, "bf16")
    # fp32 / small heads too
    w = synth.make_varlen([70, 500, 33], 4, 2, 64, seed=78, dtype="fp32")
    gp, op = _params(m, oracle, "fp32", 4, 2, 64, n_init=1, n_local=2, topk_total=4, dense_threshold=100)
    _run_prefill_case(m, oracle, w, gp, op, "fp32")


@pytest.mark.parametrize("dtype,hq,hkv,d", [("bf16", 32, 2, 128), ("fp32", 4, 1, 64)])
def test_decode_matches_oracle_and_prefill_row(m, oracle, dtype, hq, hkv, d):
    ctx = [3000, 641, 64, 33, 5, 2049, 1]
    w = synth.make_decode(ctx, hq, hkv, d, seed=31, dtype=dtype, max_len=3008)
    gp, op = _params(m, oracle, dtype, hq, hkv, d, n_init=1, n_local=2, topk_total=8)
    q, kc_, vc_ = to_dev(w["q"], dtype), to_dev(w["k_cache"], dtype), to_dev(w["v_cache"], dtype)
    B = len(ctx)
    max_nc = oracle.num_cmp(3008, op)
    kcc = torch.zeros((B, hkv, max_nc, d), dtype=torch.float32, device="cuda")
    for b, L in enumerate(ctx):      # compressed-key cache built by the library's own stage 1
        kcb, _ = m.compress_k(gp, kc_[b, :, :L], [0, L])
        nc = oracle.num_cmp(L, op)
        kcc[b, :, :nc] = kcb[:, :nc]
    out, lse, idx = m.sparse_decode(gp, q, kc_, vc_, kcc, ctx)
    torch.cuda.synchronize()
    ref = oracle.decode(w["q"], w["k_cache"], w["v_cache"], ctx, op)
    idx = to_np(idx)
    G = hq // hkv
    for b, L in enumerate(ctx):
        pos = np.array([L - 1], np.int32)
        for h in range(hkv):
            Kh = w["k_cache"][b, h, :L]
            sh = oracle.block_scores(w["q"][b:b + 1, h * G:(h + 1) * G], pos, oracle.compress_k(Kh, op), op)
            io, co = oracle.topk_blocks(sh, pos, op, return_cmp=True)
            check_selection(idx[b, h][None], io, co, pos, op.n_init, op.n_local)
            O, Ls = oracle.sparse_attn(w["q"][b:b + 1, h * G:(h + 1) * G], pos, Kh, w["v_cache"][b, h, :L],
                                       idx[b, h][None], op)
            assert_out_close(to_np(out)[b, h * G:(h + 1) * G], O[0], dtype, "decode out | GPU selection")
            np.testing.assert_allclose(to_np(lse)[b, h * G:(h + 1) * G], Ls[0], atol=2e-3 if dtype == "bf16" else 1e-4)
    # end to end, per (sequence, KV head): wherever the list equals the oracle's, so must the output
    n_same = 0
    for b in range(B):
        for h in range(hkv):
            if np.array_equal(idx[b, h], ref["idx"][b, h]):
                n_same += 1
                assert_out_close(to_np(out)[b, h * G:(h + 1) * G], ref["out"][b, h * G:(h + 1) * G], dtype, "decode out")
    assert n_same >= B * hkv - 1
    # decode == last row of the library's own prefill on the same sequence
    L = ctx[0]
    q_full = torch.zeros((L, hq, d), dtype=q.dtype, device="cuda")
    q_full[L - 1] = q[0]
    pre = m.sparse_prefill(gp, q_full, kc_[0, :, :L], vc_[0, :, :L], [0, L])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_np(pre["block_idx"])[:, L - 1], idx[0])
    assert_out_close(to_np(pre["out"])[L - 1], to_np(out)[0], dtype, "decode vs prefill row")


def _check_decode(m, oracle, w, ctx, gp, op, dtype):
    hq, hkv, d = gp.num_q_heads, gp.num_kv_heads, gp.head_dim
    G = hq // hkv
    q, kc_, vc_ = to_dev(w["q"], dtype), to_dev(w["k_cache"], dtype), to_dev(w["v_cache"], dtype)
    B = len(ctx)
    lmax = w["k_cache"].shape[2]
    max_nc = max(oracle.num_cmp(lmax, op), 1)
    kcc = torch.zeros((B, hkv, max_nc, d), dtype=torch.float32, device="cuda")
    for b, L in enumerate(ctx):
        nc = oracle.num_cmp(int(L), op)
        if nc:
            kcb, _ = m.compress_k(gp, kc_[b, :, :int(L)], [0, int(L)])
            kcc[b, :, :nc] = kcb[:, :nc]
    out, lse, idx = m.sparse_decode(gp, q, kc_, vc_, kcc, ctx)
    torch.cuda.synchronize()
    out, lse, idx = to_np(out), to_np(lse), to_np(idx)
    n_sparse = 0
    for b, L in enumerate(ctx):
        L = int(L)
        pos = np.array([L - 1], np.int32)
        for h in range(hkv):
            Qh = w["q"][b:b + 1, h * G:(h + 1) * G]
            Kh, Vh = w["k_cache"][b, h, :L], w["v_cache"][b, h, :L]
            if L < op.dense_threshold:
                assert np.all(idx[b, h] == -1)
                O, Ls = oracle.dense_attn(Qh, pos, Kh, Vh, op)
            else:
                n_sparse += 1
                sh = oracle.block_scores(Qh, pos, oracle.compress_k(Kh, op), op,
                                         kc2=oracle.compress_k(Kh, op, level=2) if op.lse_mode else None)
                io, co = oracle.topk_blocks(sh, pos, op, return_cmp=True)
                check_selection(idx[b, h][None], io, co, pos, op.n_init, op.n_local)
                O, Ls = oracle.sparse_attn(Qh, pos, Kh, Vh, idx[b, h][None], op)
            assert_out_close(out[b, h * G:(h + 1) * G], O[0], dtype, "decode out | GPU selection")
            np.testing.assert_allclose(lse[b, h * G:(h + 1) * G], Ls[0], atol=2e-3 if dtype == "bf16" else 1e-4)
    return n_sparse


def test_compress_k_append_keeps_the_decode_cache_current(m, oracle):
    """Growing caches: the appended compressed keys must equal stage 1 on the grown sequence (oracle), rows that
    already existed must stay untouched, and steps that complete no window must write nothing."""
    for dtype, hkv, d in (("bf16", 2, 128), ("fp32", 2, 64)):
        gp, op = _params(m, oracle, dtype, 2 * hkv, hkv, d)
        prev = [0, 31, 47, 48, 1000, 500]
        ctx = [40, 32, 47, 200, 1001, 564]
        w = synth.make_decode(ctx, 2 * hkv, hkv, d, seed=21, dtype=dtype, max_len=1100)
        kcache = to_dev(w["k_cache"], dtype)
        max_nc = oracle.num_cmp(1100, op)
        kcc = torch.full((len(ctx), hkv, max_nc, d), 7.0, dtype=torch.float32, device="cuda")
        for b, L in enumerate(prev):                       # the cache as it stood at prev
            nc = oracle.num_cmp(L, op)
            if nc:
                kcb, _ = m.compress_k(gp, kcache[b, :, :L], [0, L])
                kcc[b, :, :nc] = kcb[:, :nc]
        before = kcc.clone()
        m.compress_k_append(gp, kcache, kcc, prev, ctx)
        torch.cuda.synchronize()
        got, before = to_np(kcc), to_np(before)
        for b, (L0, L1) in enumerate(zip(prev, ctx)):
            n0, n1 = oracle.num_cmp(L0, op), oracle.num_cmp(L1, op)
            for h in range(hkv):
                want = oracle.compress_k(w["k_cache"][b, h, :L1], op)
                np.testing.assert_allclose(got[b, h, n0:n1], want[n0:n1], rtol=0, atol=2e-6)
                np.testing.assert_array_equal(got[b, h, :n0], before[b, h, :n0])
                np.testing.assert_array_equal(got[b, h, n1:], before[b, h, n1:])


def test_decode_dense_switch_and_ragged(m, oracle):
    """Decode with sequences on both sides of the dense threshold, partial last blocks, tiny contexts."""
    ctx = [1, 2, 31, 32, 63, 64, 65, 127, 700, 1024, 1023, 2500, 4097]
    for dtype, hq, hkv, d in [("bf16", 32, 2, 128), ("fp32", 4, 2, 64)]:
        w = synth.make_decode(ctx, hq, hkv, d, seed=91, dtype=dtype, max_len=4160)
        gp, op = _params(m, oracle, dtype, hq, hkv, d, n_init=1, n_local=2, topk_total=9, dense_threshold=1024)
        assert _check_decode(m, oracle, w, ctx, gp, op, dtype) == 3 * hkv


def test_decode_many_pairs_launch_shape(m, oracle):
    """With more (sequence, KV head) pairs than one workgroup per CU the attend kernel of the three-stage form runs
    four blocks per workgroup instead of eight (another split count, another partial layout): 40 sequences x 2 KV
    heads x 7 splits.  Mixed lengths, two of them below the dense threshold."""
    rng = np.random.default_rng(404)
    ctx = [int(x) for x in rng.integers(1100, 6000, size=38)] + [700, 64]
    w = synth.make_decode(ctx, 32, 2, 128, seed=92, dtype="bf16", max_len=6016)
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=8, topk_total=64, dense_threshold=1024)
    assert _check_decode(m, oracle, w, ctx, gp, op, "bf16") == 38 * 2


def test_decode_selection_with_tied_scores(m, oracle):
    """Key caches that repeat with a period of one or two blocks: the pooled scores of the blocks of one kind are equal
    bit for bit (each logit is a dot product of the same numbers in the same order), so the k-th largest score is
    shared by many blocks and Eq. 2's arg-max takes the lower block numbers among them -- the oracle's repeated arg-max
    and the decode kernel's radix select + ordered emission must then give the same list, element for element.  With a
    period of four blocks there are three or four kinds: the best is taken whole and only the first few of the next."""
    hq, hkv, d = 32, 2, 128
    ctx = [5000, 2300, 4100]
    for period, topk_total in ((64, 12), (256, 30)):
        w = synth.make_decode(ctx, hq, hkv, d, seed=93, dtype="bf16", max_len=5056)
        kc = w["k_cache"]
        for b, L in enumerate(ctx):
            kc[b, :, :L] = np.tile(kc[b, :, :period], (1, (L + period - 1) // period, 1))[:, :L]
        gp, op = _params(m, oracle, "bf16", hq, hkv, d, n_init=1, n_local=2, topk_total=topk_total)
        q, kc_, vc_ = to_dev(w["q"], "bf16"), to_dev(kc, "bf16"), to_dev(w["v_cache"], "bf16")
        kcc = torch.zeros((len(ctx), hkv, oracle.num_cmp(5056, op), d), dtype=torch.float32, device="cuda")
        for b, L in enumerate(ctx):
            kcb, _ = m.compress_k(gp, kc_[b, :, :L], [0, L])
            kcc[b, :, :oracle.num_cmp(L, op)] = kcb[:, :oracle.num_cmp(L, op)]
        out, lse, idx = m.sparse_decode(gp, q, kc_, vc_, kcc, ctx)
        torch.cuda.synchronize()
        ref = oracle.decode(w["q"], kc, w["v_cache"], ctx, op)
        idx = to_np(idx)
        # the ties are real: among the blocks the top-k chooses from there are far fewer distinct scores than blocks
        G = hq // hkv
        pos = np.array([ctx[0] - 1], np.int32)
        sh = oracle.block_scores(w["q"][0:1, 0:G], pos, oracle.compress_k(kc[0, 0, :ctx[0]], op), op)
        _, co = oracle.topk_blocks(sh, pos, op, return_cmp=True)
        live = np.asarray(co)[0, 1:(ctx[0] - 1) // 64 - 2]
        assert len(np.unique(live)) <= period // 64
        np.testing.assert_array_equal(idx, ref["idx"])
        assert_out_close(to_np(out), ref["out"], "bf16", "decode out, tied scores")


def test_decode_c4_full_shape(m, oracle):
    """Workload C4 at full size: batch 16, context lengths uniform in [16384, 65536], top-k 64."""
    cfg = synth.CONFIGS["C4"]
    ctx = synth.draw_ctx_lens(cfg.batch, cfg.ctx_lo, cfg.ctx_hi, cfg.seed)
    w = synth.make_config(cfg, ctx_lens=ctx)
    gp, op = m.Params.from_config(cfg), oracle.Params.from_config(cfg)
    assert _check_decode(m, oracle, w, ctx, gp, op, "bf16") == 32


def test_empty_batch_and_empty_sequences(m, oracle):
    gp, op = _params(m, oracle, "bf16", 32, 2, 128)
    q = torch.zeros((0, 32, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((2, 0, 128), dtype=torch.bfloat16, device="cuda")
    res = m.sparse_prefill(gp, q, k, k, [0])
    assert res["out"].shape[0] == 0
    # a zero-length sequence in the middle of a batch
    w = synth.make_varlen([130, 200], 4, 2, 64, seed=3, dtype="fp32")
    cu3 = np.array([0, 130, 130, 330], np.int32)
    gp, op = _params(m, oracle, "fp32", 4, 2, 64, n_init=1, n_local=2, topk_total=4)
    q, k, v = (to_dev(w[x], "fp32") for x in ("q", "k", "v"))
    a = m.sparse_prefill(gp, q, k, v, w["cu_seqlens"])
    b = m.sparse_prefill(gp, q, k, v, cu3)
    torch.cuda.synchronize()
    assert torch.equal(a["out"], b["out"]) and torch.equal(a["block_idx"], b["block_idx"])


def test_token_major_kv_layout_gives_identical_results(m, oracle):
    """K and V may be addressed with any (token, head) strides: a token-major [T, hkv, d] buffer viewed as
    [hkv, T, d] must give bit-identical results to the head-major copy, in prefill (MFMA and generic kernels)
    and in decode (cache stored [B, Lmax, hkv, d])."""
    for dtype, hq, hkv, d, n in (("bf16", 32, 2, 128, 1500), ("fp32", 4, 2, 64, 700)):
        w = synth.make_prefill(n, hq, hkv, d, seed=41, dtype=dtype)
        gp, _ = _params(m, oracle, dtype, hq, hkv, d, n_init=1, n_local=2, topk_total=9)
        q, k, v = (to_dev(w[x], dtype) for x in ("q", "k", "v"))
        kt = k.permute(1, 0, 2).contiguous().permute(1, 0, 2)         # same values, token-major storage
        vt = v.permute(1, 0, 2).contiguous().permute(1, 0, 2)
        assert kt.stride() == (d, hkv * d, 1)
        a = m.sparse_prefill(gp, q, k, v, w["cu_seqlens"])
        b = m.sparse_prefill(gp, q, kt, vt, w["cu_seqlens"])
        torch.cuda.synchronize()
        for key in ("out", "lse", "block_idx", "kc"):
            assert torch.equal(a[key], b[key]), (dtype, key)
        da, _ = m.dense_attn_fwd(gp, q, k, v, w["cu_seqlens"])
        db, _ = m.dense_attn_fwd(gp, q, kt, vt, w["cu_seqlens"])
        assert torch.equal(da, db)
    ctx = [900, 65, 3000]
    dw = synth.make_decode(ctx, 32, 2, 128, seed=42, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=2, topk_total=9)
    q, kc_, vc_ = to_dev(dw["q"], "bf16"), to_dev(dw["k_cache"], "bf16"), to_dev(dw["v_cache"], "bf16")
    kcc = torch.zeros((3, 2, max(oracle.num_cmp(3000, op), 1), 128), dtype=torch.float32, device="cuda")
    m.compress_k_append(gp, kc_, kcc, [0, 0, 0], ctx)
    kt = kc_.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)     # stored [B, Lmax, hkv, d]
    vt = vc_.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    kcc2 = torch.zeros_like(kcc)
    m.compress_k_append(gp, kt, kcc2, [0, 0, 0], ctx)
    oa, la, ia = m.sparse_decode(gp, q, kc_, vc_, kcc, ctx)
    ob, lb, ib = m.sparse_decode(gp, q, kt, vt, kcc2, ctx)
    torch.cuda.synchronize()
    assert torch.equal(kcc, kcc2) and torch.equal(oa, ob) and torch.equal(la, lb) and torch.equal(ia, ib)


def test_shifted_pool_window_and_lse_approximation_with_switch(m, oracle):
    """pool_pad = 1 (the shifted reading of Eq. 6) through the MFMA path, and lse_mode 1 on a packed batch with
    sequences on both sides of the dense threshold."""
    w = synth.make_prefill(2100, 32, 2, 128, seed=43, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=2, topk_total=11, pool_pad=1)
    _run_prefill_case(m, oracle, w, gp, op, "bf16")
    w = synth.make_varlen((300, 150, 1200, 640), 32, 2, 128, seed=44, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=3, topk_total=8, dense_threshold=600, lse_mode=1)
    _run_prefill_case(m, oracle, w, gp, op, "bf16")


def test_determinism(m, oracle):
    """The forward path has no atomics on floats anywhere: two runs give bitwise identical results (a difference
    would mean a race).  In the backward, dQ is likewise reproducible bit for bit; dK and dV are summed with the
    L2's float atomics, so their last bits may differ between runs (bounded below, relative to the largest
    gradient)."""
    w = synth.make_prefill(3000, 32, 2, 128, seed=55, dtype="bf16")
    gp, _ = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=8, topk_total=16)
    q, k, v = (to_dev(w[x], "bf16") for x in ("q", "k", "v"))
    a = m.sparse_prefill(gp, q, k, v, [0, 3000])
    b = m.sparse_prefill(gp, q, k, v, [0, 3000])
    torch.cuda.synchronize()
    for key in ("out", "lse", "block_idx", "kc"):
        assert torch.equal(a[key], b[key]), key
    dout = torch.randn_like(q)
    g1 = m.sparse_attn_bwd(gp, q, k, v, a["block_idx"], a["out"], a["lse"], dout, [0, 3000])
    g2 = m.sparse_attn_bwd(gp, q, k, v, a["block_idx"], a["out"], a["lse"], dout, [0, 3000])
    torch.cuda.synchronize()
    assert torch.equal(g1[0], g2[0]), "dq"
    for x, y, name in ((g1[1], g2[1], "dk"), (g1[2], g2[2], "dv")):
        assert float((x - y).abs().max()) <= 1e-5 * max(1.0, float(x.abs().max())), name


# ------------------------------------------------------------------------ max-pooling fused into the score kernel
def _check_fused_pool(m, oracle, w, gp, op, dtype):
    """The pooled entry points against (a) the two-stage GPU path, bit for bit, and (b) the oracle's Eq. 6."""
    cu = w["cu_seqlens"]
    T, hq, d = w["q"].shape
    hkv = w["k"].shape[0]
    G = hq // hkv
    q, k, v = (to_dev(w[x], dtype) for x in ("q", "k", "v"))
    two = m.sparse_prefill(gp, q, k, v, cu)
    # poison the pooled buffer: entries the kernel must not define stay NaN and must not influence the selection
    si = m.SeqInfo(cu)
    kc, cu_c = two["kc"], two["cu_seqlens_c"]
    max_len = int(np.diff(cu).max()) if len(cu) > 1 else 0
    nb = max(1, -(-max_len // 64))
    s_cmp = torch.full((hkv, T, nb + 3), float("nan"), dtype=torch.float32, device="cuda")
    m.block_scores_pooled(gp, q, kc, si, cu_c, out=s_cmp)
    idx_f = m.topk_pooled(gp, s_cmp, si)
    torch.cuda.synchronize()
    sh_g, sc_g = to_np(two["s_shared"]), to_np(s_cmp)
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if b - a < op.dense_threshold or b == a:
            assert np.all(np.isnan(sc_g[:, a:b]))
            continue
        pos = np.arange(b - a, dtype=np.int32)
        for h in range(hkv):
            kc_o = oracle.compress_k(w["k"][h, a:b], op)
            sh_o = oracle.block_scores(w["q"][a:b, h * G:(h + 1) * G], pos, kc_o, op,
                                       kc2=oracle.compress_k(w["k"][h, a:b], op, level=2) if op.lse_mode else None)
            _, cmp_o = oracle.topk_blocks(sh_o, pos, op, return_cmp=True)
            for t in range(b - a):
                vis = oracle.visible_cmp(t, op)
                row = sc_g[h, a + t]
                defined = np.array([j <= t // 64 and max(op.pool_stride * j - op.pool_pad, 0) < vis
                                    for j in range(row.shape[0])])
                assert np.all(np.isnan(row[~defined])), (s, h, t)
                js = np.nonzero(defined)[0]
                if len(js) == 0:
                    continue
                # (a) exactly the max over the window of the scores the unfused kernel stores
                want = np.array([sh_g[h, a + t, max(op.pool_stride * j - op.pool_pad, 0):
                                      min(op.pool_stride * j - op.pool_pad + op.pool_len, vis)].max() for j in js])
                np.testing.assert_array_equal(row[js], want)
                # (b) the oracle's pooled scores
                np.testing.assert_allclose(row[js], cmp_o[t, js], rtol=5e-4, atol=1e-7)
    np.testing.assert_array_equal(to_np(idx_f), to_np(two["block_idx"]))


@pytest.mark.parametrize("pool_pad", [0, 1])
@pytest.mark.parametrize("lse_mode", [0, 1])
def test_fused_pooling_paper_head_shape(m, oracle, pool_pad, lse_mode):
    """Matrix-core score kernel with Eq. 6 fused: several key tiles, ragged tails, lengths at tile boundaries
    (1055 = 64 visible keys + 31, 2079 = 128 + 31 for the last token), a length below the first window."""
    lens = [1055, 20, 2079, 700, 1500]
    w = synth.make_varlen(lens, 32, 2, 128, seed=4242 + pool_pad + 2 * lse_mode, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=2, topk_total=7, pool_pad=pool_pad, lse_mode=lse_mode)
    _check_fused_pool(m, oracle, w, gp, op, "bf16")


@pytest.mark.parametrize("pool", [(5, 4, 0), (5, 4, 1), (3, 2, 0), (8, 4, 2), (1, 1, 0)])
def test_fused_pooling_generic_kernel(m, oracle, pool):
    """fp32 / small heads take the one-row-per-workgroup kernel, which accepts any pooling window."""
    pl, ps, pad = pool
    w = synth.make_varlen([900, 31, 333], 4, 2, 64, seed=977 + pl, dtype="fp32")
    gp, op = _params(m, oracle, "fp32", 4, 2, 64, n_init=1, n_local=1, topk_total=5, pool_len=pl, pool_stride=ps,
                     pool_pad=pad)
    _check_fused_pool(m, oracle, w, gp, op, "fp32")


def test_fused_pooling_with_dense_switch_and_full_path(m, oracle):
    """Sequences below the threshold get no pooled scores and an all -1 list; sparse_prefill(fused_pool=True)
    returns the same output as the two-stage path."""
    lens = [300, 1200, 100]
    w = synth.make_varlen(lens, 32, 2, 128, seed=31, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=2, topk_total=6, dense_threshold=512)
    _check_fused_pool(m, oracle, w, gp, op, "bf16")
    q, k, v = (to_dev(w[x], "bf16") for x in ("q", "k", "v"))
    a = m.sparse_prefill(gp, q, k, v, w["cu_seqlens"])
    b = m.sparse_prefill(gp, q, k, v, w["cu_seqlens"], fused_pool=True)
    torch.cuda.synchronize()
    assert torch.equal(a["block_idx"], b["block_idx"]) and torch.equal(a["out"], b["out"]) and torch.equal(a["lse"], b["lse"])


# ------------------------------------------------------------------------------- stage 3 alone on long rows
@pytest.mark.parametrize("kind", ["continuous", "quantised", "mostly_zero", "one_level"])
@pytest.mark.parametrize("topk_total", [64, 96, 200])
def test_topk_long_rows_bit_exact(m, oracle, kind, topk_total):
    """Rows of more than 256 blocks narrow the search to a candidate set first; rows where that cannot work (mass
    ties, too few positive scores, more than 64 to pick) take the general path.  Both must give the oracle's list
    bit for bit, from scores per compressed key and from pooled scores."""
    n, hkv = 21000, 1
    rng = np.random.default_rng(500 + len(kind) + topk_total)
    gp, op = _params(m, oracle, "bf16", 16, hkv, 128, n_init=1, n_local=8 if topk_total != 96 else 32,
                     topk_total=topk_total)
    nc = oracle.num_cmp(n, op)
    rs = (nc + 3) // 4 * 4
    s = rng.random((hkv, n, rs), dtype=np.float32)
    if kind == "quantised":
        s = np.floor(s * 8) / 8
    elif kind == "mostly_zero":
        s = np.where(rng.random(s.shape) < 0.004, s, 0).astype(np.float32)
    elif kind == "one_level":
        s[:] = 0.25
    s_d = torch.from_numpy(s).cuda()
    si = m.SeqInfo([0, n])
    idx_g = to_np(m.topk_blocks(gp, s_d, si))
    rows = np.unique(np.concatenate([np.arange(0, n, 97), np.arange(16000, 17000), np.arange(n - 300, n)])).astype(np.int32)
    idx_o, cmp_o = oracle.topk_blocks(s[0, rows], rows, op, return_cmp=True)
    np.testing.assert_array_equal(idx_g[0, rows], idx_o)
    # the same selection from pooled scores: S^cmp as the oracle computes it, NaN where undefined
    nb = -(-n // 64)
    sc = np.full((hkv, n, nb), np.nan, dtype=np.float32)
    for r, t in enumerate(rows):
        vis = oracle.visible_cmp(int(t), op)
        for j in range(t // 64 + 1):
            if max(4 * j, 0) < vis:
                sc[0, t, j] = cmp_o[r, j]
    idx_p = to_np(m.topk_pooled(gp, torch.from_numpy(sc).cuda(), si))
    np.testing.assert_array_equal(idx_p[0, rows], idx_o)


# ----------------------------------------------------------------------------- gradients of stage 4
def _check_backward(m, oracle, w, gp, op, dtype, dense_all=False, sel_bitmap_max_bytes=512 << 20):
    """dQ, dK, dV of the GPU (through the C ABI, from the GPU's own forward outputs and selection) against the
    oracle's float64 gradients for the same selection.  Errors are measured relative to the largest magnitude of
    each gradient (at least 0.1; inputs are O(1)): fp32 data max 2e-4 / mean 5e-5 (fast exponentials, float accumulation over up to n rows); bf16 data max 2e-2 /
    mean 2e-3, the forward bar, because Delta = <dO, O> is formed from the bf16-rounded O and dQ is stored in bf16."""
    cu = w["cu_seqlens"]
    T, hq, d = w["q"].shape
    hkv = w["k"].shape[0]
    G = hq // hkv
    q, k, v = (to_dev(w[x], dtype) for x in ("q", "k", "v"))
    rng = np.random.default_rng(12345 + T)
    dout_np = synth.round_to_bf16(rng.standard_normal((T, hq, d)).astype(np.float32)) if dtype == "bf16" else \
        rng.standard_normal((T, hq, d)).astype(np.float32)
    dout = to_dev(dout_np, dtype)
    si = m.SeqInfo(cu)
    if dense_all:
        out, lse = m.dense_attn_fwd(gp, q, k, v, si)
        idx_d = None
    else:
        res = m.sparse_prefill(gp, q, k, v, si)
        out, lse, idx_d = res["out"], res["lse"], res["block_idx"]
    dq, dk, dv = m.sparse_attn_bwd(gp, q, k, v, idx_d, out, lse, dout, si, sel_bitmap_max_bytes=sel_bitmap_max_bytes)
    dq2, dk2, dv2 = m.sparse_attn_bwd(gp, q, k, v, idx_d, out, lse, dout, si, sel_bitmap_max_bytes=sel_bitmap_max_bytes)
    torch.cuda.synchronize()
    assert torch.equal(dq, dq2)                                  # no atomics on this path
    dq_g, dk_g, dv_g = to_np(dq), to_np(dk), to_np(dv)
    idx_g = None if idx_d is None else to_np(idx_d)
    max_tol, mean_tol = (2e-2, 2e-3) if dtype == "bf16" else (2e-4, 5e-5)
    worst = 0.0
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        if a == b:
            continue
        pos = np.arange(b - a, dtype=np.int32)
        dense = dense_all or (b - a) < op.dense_threshold
        for h in range(hkv):
            sel = None if dense else idx_g[h, a:b]
            dQ, dK, dV = oracle.attn_bwd(w["q"][a:b, h * G:(h + 1) * G], pos, w["k"][h, a:b], w["v"][h, a:b], sel,
                                         dout_np[a:b, h * G:(h + 1) * G], op)
            for name, got, ref in (("dq", dq_g[a:b, h * G:(h + 1) * G], dQ), ("dk", dk_g[h, a:b], dK),
                                   ("dv", dv_g[h, a:b], dV)):
                # (a single visible key gives dz = 0 exactly: dQ = dK = 0, so the scale has a floor)
                scale = max(float(np.abs(ref).max()), 0.1)
                err = np.abs(got.astype(np.float64) - ref) / scale
                assert err.max() <= max_tol and err.mean() <= mean_tol, (name, s, h, err.max(), err.mean())
                worst = max(worst, float(err.max()))
    # float atomics: a second run may differ in the last bits only
    np.testing.assert_allclose(to_np(dk2), dk_g, rtol=0, atol=1e-5 * max(1.0, float(np.abs(dk_g).max())))
    np.testing.assert_allclose(to_np(dv2), dv_g, rtol=0, atol=1e-5 * max(1.0, float(np.abs(dv_g).max())))
    return worst


@pytest.mark.parametrize("n", [1, 65, 200, 700])
def test_backward_fp32_small_heads(m, oracle, n):
    w = synth.make_prefill(n, 4, 2, 64, seed=300 + n, dtype="fp32")
    gp, op = _params(m, oracle, "fp32", 4, 2, 64, n_init=1, n_local=1, topk_total=3)
    _check_backward(m, oracle, w, gp, op, "fp32")


def test_backward_fp32_group_of_16_d128_and_dense(m, oracle):
    w = synth.make_prefill(330, 16, 1, 128, seed=311, dtype="fp32")
    gp, op = _params(m, oracle, "fp32", 16, 1, 128, n_init=1, n_local=2, topk_total=4)
    _check_backward(m, oracle, w, gp, op, "fp32")
    _check_backward(m, oracle, w, gp, op, "fp32", dense_all=True)


def test_backward_bf16_paper_head_shape_varlen_with_switch(m, oracle):
    """Paper head shape in bf16, packed sequences on both sides of the dense threshold, one crossing a chunk of
    256 tokens several times."""
    w = synth.make_varlen([300, 50, 900], 32, 2, 128, seed=312, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=2, topk_total=5, dense_threshold=256)
    _check_backward(m, oracle, w, gp, op, "bf16")


@pytest.mark.parametrize("n", [1, 63, 64, 129, 2500])
def test_backward_bf16_matrix_core_path(m, oracle, n):
    """The matrix-core backward (bf16, 16 heads per KV head, d 128): ragged lengths, a sequence longer than one
    2048-token chunk of the dK/dV kernel, sparse and dense."""
    w = synth.make_prefill(n, 32, 2, 128, seed=320 + n, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=2, topk_total=6)
    _check_backward(m, oracle, w, gp, op, "bf16")
    if n <= 129:
        _check_backward(m, oracle, w, gp, op, "bf16", dense_all=True)


@pytest.mark.parametrize("case", range(10))
def test_seeded_random_configurations(m, oracle, case):
    """Randomly drawn (but seeded, hence repeatable) workloads on the matrix-core path: packed lengths on both
    sides of the switch, selection budgets, pooling shift and the LSE Approximation, every stage against the
    oracle.  Complements the hand-picked cases above with combinations nobody thought of."""
    rng = np.random.default_rng(9000 + case)
    nseq = int(rng.integers(1, 5))
    lens = [int(x) for x in rng.choice([1, 17, 31, 32, 63, 64, 65, 127, 129, 300, 511, 777, 1200, 1700], size=nseq)]
    n_init = int(rng.integers(0, 3))
    n_local = int(rng.integers(1, 5))
    topk_total = n_init + n_local + int(rng.integers(0, 8))
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=n_init, n_local=n_local, topk_total=topk_total,
                     dense_threshold=int(rng.choice([0, 64, 400, 1000])), pool_pad=int(rng.integers(0, 2)),
                     lse_mode=int(rng.integers(0, 2)))
    w = synth.make_varlen(lens, 32, 2, 128, seed=9100 + case, dtype="bf16")
    _run_prefill_case(m, oracle, w, gp, op, "bf16")
    # the fused-pooling form of stages 2-3 selects the same blocks
    q, k, v = (to_dev(w[x], "bf16") for x in ("q", "k", "v"))
    two = m.sparse_prefill(gp, q, k, v, w["cu_seqlens"])
    fused = m.sparse_prefill(gp, q, k, v, w["cu_seqlens"], fused_pool=True)
    torch.cuda.synchronize()
    assert torch.equal(two["block_idx"], fused["block_idx"]) and torch.equal(two["out"], fused["out"])


@pytest.mark.parametrize("case", range(6))
def test_seeded_random_decode_configurations(m, oracle, case):
    """The decode step on randomly drawn (seeded) batches: context lengths around block, window and switch
    boundaries, selection budgets, pooling shift and the LSE Approximation, against the oracle."""
    rng = np.random.default_rng(9500 + case)
    ctx = [int(x) for x in rng.choice([1, 2, 31, 32, 33, 64, 65, 128, 200, 513, 1000, 2047, 2048, 2049, 3333, 5000],
                                      size=int(rng.integers(1, 7)))]
    n_init = int(rng.integers(0, 3))
    n_local = int(rng.integers(1, 5))
    topk_total = n_init + n_local + int(rng.integers(0, 12))
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=n_init, n_local=n_local, topk_total=topk_total,
                     dense_threshold=int(rng.choice([0, 100, 1500])), pool_pad=int(rng.integers(0, 2)),
                     lse_mode=int(rng.integers(0, 2)))
    w = synth.make_decode(ctx, 32, 2, 128, seed=9600 + case, dtype="bf16", max_len=(max(ctx) + 63) // 64 * 64)
    _check_decode(m, oracle, w, ctx, gp, op, "bf16")


@pytest.mark.parametrize("case", range(5))
def test_seeded_random_backward_configurations(m, oracle, case):
    """Gradients of stage 4 on randomly drawn (seeded) packed workloads, matrix-core path."""
    rng = np.random.default_rng(9700 + case)
    lens = [int(x) for x in rng.choice([1, 33, 64, 65, 130, 257, 600, 1100], size=int(rng.integers(1, 4)))]
    n_init = int(rng.integers(0, 3))
    n_local = int(rng.integers(1, 4))
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=n_init, n_local=n_local,
                     topk_total=n_init + n_local + int(rng.integers(0, 6)), dense_threshold=int(rng.choice([0, 100, 500])))
    w = synth.make_varlen(lens, 32, 2, 128, seed=9800 + case, dtype="bf16")
    _check_backward(m, oracle, w, gp, op, "bf16")


def test_backward_without_selection_bitmap(m, oracle):
    """The dK/dV kernel normally reads which tokens selected a block from a bitmap built by a pre-pass; a workspace
    without room for the bitmap makes it search the tokens' lists instead.  Take that route and check it the same
    way."""
    w = synth.make_varlen([300, 50, 2300], 32, 2, 128, seed=331, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=2, topk_total=6, dense_threshold=256)
    assert m.workspace_bytes(m.OP_SPARSE_ATTN_BWD, gp, 3, 2650, 2300) > m.workspace_bytes(m.OP_SPARSE_ATTN_BWD_MIN, gp, 3, 2650, 2300)
    _check_backward(m, oracle, w, gp, op, "bf16", sel_bitmap_max_bytes=0)


def test_decode_step_replays_from_a_hip_graph(m, oracle):
    """The decode call allocates nothing and enqueues only kernels on the caller's stream, so a serving loop can
    capture it once and replay it.  Replays (with eager work and synchronisations in between, and with the inputs
    changed in place) must reproduce the eager results bit for bit."""
    ctx = [3000, 641, 64, 2049]
    w = synth.make_decode(ctx, 32, 2, 128, seed=41, dtype="bf16", max_len=3008)
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=2, topk_total=8)
    q, kc_, vc_ = to_dev(w["q"], "bf16"), to_dev(w["k_cache"], "bf16"), to_dev(w["v_cache"], "bf16")
    B = len(ctx)
    kcc = torch.zeros((B, 2, oracle.num_cmp(3008, op), 128), dtype=torch.float32, device="cuda")
    for b, L in enumerate(ctx):
        kcb, _ = m.compress_k(gp, kc_[b, :, :L], [0, L])
        kcc[b, :, :kcb.shape[1]] = kcb
    di = m.DecodeInfo(ctx)
    ws = torch.empty(m.decode_workspace_bytes(gp, B, di.max_ctx), dtype=torch.uint8, device="cuda")
    out_e, lse_e, idx_e = m.sparse_decode(gp, q, kc_, vc_, kcc, di, workspace=ws)          # eager (also warms up)
    torch.cuda.synchronize()
    q_s = q.clone()
    out_g, lse_g, idx_g = torch.empty_like(out_e), torch.empty_like(lse_e), torch.empty_like(idx_e)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        m.sparse_decode(gp, q_s, kc_, vc_, kcc, di, workspace=ws, out=out_g, lse=lse_g, idx=idx_g)
    q2 = (q.float() * 0.5 + 0.25).to(torch.bfloat16)
    out_e2, lse_e2, idx_e2 = m.sparse_decode(gp, q2, kc_, vc_, kcc, di, workspace=ws.clone())
    torch.cuda.synchronize()
    for rep in range(4):
        src, ref = (q, (out_e, lse_e, idx_e)) if rep % 2 == 0 else (q2, (out_e2, lse_e2, idx_e2))
        q_s.copy_(src)
        out_g.zero_(); lse_g.zero_(); idx_g.zero_()
        junk = torch.randn(1 << 16, device="cuda").sum()                                      # eager work in between
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_g, ref[0]) and torch.equal(lse_g, ref[1]) and torch.equal(idx_g, ref[2]), rep
        assert torch.isfinite(junk)


def test_prefill_calls_replay_from_a_hip_graph(m, oracle):
    """The four prefill calls allocate nothing (every scratch buffer is the caller's) and only enqueue kernels, so
    they can be captured once and replayed.  Replays, with eager work and synchronisations in between and the inputs
    changed in place, must reproduce the eager results bit for bit."""
    n = 3000
    w = synth.make_prefill(n, 32, 2, 128, seed=91, dtype="bf16")
    gp, _ = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=8, topk_total=16)
    q, k, v = (to_dev(w[x], "bf16") for x in ("q", "k", "v"))
    si = m.SeqInfo([0, n])
    ref1 = m.sparse_prefill(gp, q, k, v, si, fused_pool=True)                          # eager (also warms up)
    q2 = (q.float() * 0.5 + 0.125).to(torch.bfloat16)
    ref2 = m.sparse_prefill(gp, q2, k, v, si, fused_pool=True)
    torch.cuda.synchronize()
    q_s = q.clone()
    bufs = m.sparse_prefill(gp, q_s, k, v, si, fused_pool=True)                        # buffers the graph will own
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        m.sparse_prefill(gp, q_s, k, v, si, buffers=bufs, fused_pool=True)
    for rep in range(4):
        src, ref = (q, ref1) if rep % 2 == 0 else (q2, ref2)
        q_s.copy_(src)
        for key in ("out", "lse", "block_idx"):
            bufs[key].fill_(0)
        junk = torch.randn(1 << 16, device="cuda").sum()                               # eager work in between
        graph.replay()
        torch.cuda.synchronize()
        for key in ("out", "lse", "block_idx", "kc"):
            assert torch.equal(bufs[key], ref[key]), (rep, key)
        assert torch.isfinite(junk)


@pytest.mark.parametrize("cmp", [(32, 8), (32, 32), (64, 16)])
def test_other_compression_windows(m, oracle, cmp):
    """Compression windows other than the paper's (l_C1, s_C1) = (32, 16): a selection block then spans 8, 2 or 4
    compressed keys, so the on-chip pooling of the matrix-core score kernel (written for 4) must not be taken and
    the decode path must size its pooled-key row by blocks.  Prefill two-stage and fused, and decode, against the
    oracle."""
    lc, sc = cmp
    w = synth.make_prefill(1500, 32, 2, 128, seed=400 + lc + sc, dtype="bf16")
    gp, op = _params(m, oracle, "bf16", 32, 2, 128, n_init=1, n_local=2, topk_total=7, cmp_len=lc, cmp_stride=sc,
                     pool_len=64 // sc + 1, pool_stride=64 // sc)
    _run_prefill_case(m, oracle, w, gp, op, "bf16")
    _run_prefill_case(m, oracle, w, gp, op, "bf16", fused_pool=True)
    ctx = [1500, 700, 129, 40]
    wd = synth.make_decode(ctx, 32, 2, 128, seed=500 + lc + sc, dtype="bf16", max_len=1536)
    assert _check_decode(m, oracle, wd, ctx, gp, op, "bf16") >= 6
