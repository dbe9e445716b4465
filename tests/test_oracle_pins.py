"""Pins for the CPU oracle: every check compares it with something that is not itself --
closed forms, hand-worked fixtures, brute force written independently with torch/numpy in
float64, library routines (torch.softmax, scaled_dot_product_attention), and invariants the
paper's equations imply.  Citations are to arXiv 2509.24663.
"""
import math
import os

import numpy as np
import pytest
import torch

import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _read_gold(name):
    out = {}
    rows = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if ":" in line:
                k, v = line.split(":")
                out[k.strip()] = [float(x) for x in v.split()]
            else:
                rows.append([float(x) for x in line.split()])
    return out, rows


def _vis(t, lc=32, sc=16):
    return 0 if t < lc - 1 else (t - lc + 1) // sc + 1


def _small(n=300, hq=4, hkv=2, d=16, seed=7, dtype="fp32"):
    return synth.make_prefill(n, hq, hkv, d, seed=seed, dtype=dtype)


# ----------------------------------------------------------------------------- stage 1 (Eq. 3)
def test_compress_counts_and_ramp_fixture(oracle):
    p = oracle.Params()
    assert oracle.num_cmp(2048, p) == 127
    assert oracle.num_cmp(32768, p) == 2047
    assert oracle.num_cmp(131072, p) == 8191
    assert oracle.num_cmp(31, p) == 0 and oracle.num_cmp(32, p) == 1 and oracle.num_cmp(47, p) == 1
    _, rows = _read_gold("compress_ramp.txt")
    K = np.repeat(np.arange(100, dtype=np.float32)[:, None], 8, axis=1)
    kc = oracle.compress_k(K, p)
    assert kc.shape == (5, 8)
    for i, expected in rows:
        assert np.all(kc[int(i)] == np.float32(expected))


def test_compress_matches_strided_mean(oracle):
    p = oracle.Params(cmp_len=8, cmp_stride=4)
    rng = np.random.default_rng(0)
    K = rng.standard_normal((77, 5)).astype(np.float32)
    kc = oracle.compress_k(K, p)
    win = np.lib.stride_tricks.sliding_window_view(K.astype(np.float64), 8, axis=0)[::4]   # [nc, d, 8]
    np.testing.assert_allclose(kc, win.mean(-1), rtol=0, atol=1e-7)
    const = oracle.compress_k(np.full((64, 3), 2.5, np.float32), oracle.Params())
    assert np.all(const == 2.5)


# ----------------------------------------------------------------------------- stage 2 (Eq. 4, 5)
def test_scores_rows_sum_to_group_size(oracle):
    p = oracle.Params(softmax_scale=16 ** -0.5)
    w = _small()
    G = 2
    pos = np.arange(300, dtype=np.int32)
    kc = oracle.compress_k(w["k"][0], p)
    sh = oracle.block_scores(w["q"][:, :G], pos, kc, p)
    vis = np.array([_vis(t) for t in pos])
    sums = sh.astype(np.float64).sum(1)
    np.testing.assert_allclose(sums[vis > 0], G, atol=1e-5)
    assert np.all(sums[vis == 0] == 0)
    assert sh.min() >= 0 and sh.max() <= G + 1e-6
    for t in (31, 46, 47, 299):          # nothing beyond the visible prefix
        assert np.all(sh[t, _vis(t):] == 0)
        assert np.all(sh[t, :_vis(t)] > 0)


def test_scores_zero_query_is_uniform(oracle):
    p = oracle.Params()
    w = _small()
    pos = np.array([31, 100, 299], dtype=np.int32)
    kc = oracle.compress_k(w["k"][1], p)
    sh = oracle.block_scores(np.zeros((3, 2, 16), np.float32), pos, kc, p)
    for r, t in enumerate(pos):
        v = _vis(t)
        np.testing.assert_allclose(sh[r, :v], 2.0 / v, rtol=1e-6)


def test_scores_match_library_softmax(oracle):
    p = oracle.Params(softmax_scale=0.37)
    w = _small(n=260, hq=6, hkv=2, d=16, seed=3)
    G = 3
    pos = np.array([40, 133, 259], dtype=np.int32)
    kc = oracle.compress_k(w["k"][1], p)
    sh = oracle.block_scores(w["q"][pos, G:2 * G], pos, kc, p)
    # independent: windows averaged with torch, softmax from the library, in float64
    K = torch.from_numpy(w["k"][1]).double()
    kc_t = K.unfold(0, 32, 16).mean(-1)                                     # [nc, d]
    np.testing.assert_allclose(kc, kc_t.numpy(), atol=1e-6)
    for r, t in enumerate(pos):
        v = _vis(int(t))
        qt = torch.from_numpy(w["q"][t, G:2 * G]).double()                 # [G, d]
        prob = torch.softmax(0.37 * qt @ kc_t[:v].T, dim=-1).sum(0)
        np.testing.assert_allclose(sh[r, :v], prob.numpy(), rtol=2e-6, atol=1e-8)


# ----------------------------------------------------------------------------- LSE Approximation (Sec. 3.4, Eq. 7)
def _vis2(t):
    return _vis(t, 128, 64)


def test_lse_approx_coarse_keys_are_means_of_four_fine_windows(oracle):
    """K^{C2}_i = mean of 128 keys from 64 i = mean of the four disjoint 32-key windows it consists of,
    i.e. of K^{C1} rows 4i, 4i+2, 4i+4, 4i+6 (the kernels derive K^{C2} that way)."""
    p = oracle.Params(lse_mode=1)
    w = _small(n=700)
    K = w["k"][0]
    kc, kc2 = oracle.compress_k(K, p), oracle.compress_k(K, p, level=2)
    assert kc2.shape[0] == (700 - 128) // 64 + 1
    kt = torch.from_numpy(K).double().unfold(0, 128, 64).mean(-1).numpy()
    np.testing.assert_allclose(kc2, kt, atol=1e-6)
    i = np.arange(kc2.shape[0])
    np.testing.assert_allclose(kc2, (kc[4 * i] + kc[4 * i + 2] + kc[4 * i + 4] + kc[4 * i + 6]) / 4, atol=1e-6)


def test_lse_approx_constant_keys_closed_form(oracle):
    """With identical keys every logit of a head is the same number, so exp(z - lse_C2) = 1 / v2(t):
    S^shared[t, i] = G / v2(t) for every visible fine key, and 0 for rows that see no coarse key."""
    p = oracle.Params(lse_mode=1, softmax_scale=0.3)
    rng = np.random.default_rng(1)
    K = np.tile(rng.standard_normal((1, 16)).astype(np.float32), (600, 1))
    Q = rng.standard_normal((600, 3, 16)).astype(np.float32)
    pos = np.arange(600, dtype=np.int32)
    sh = oracle.block_scores(Q, pos, oracle.compress_k(K, p), p, oracle.compress_k(K, p, level=2))
    for t in (0, 31, 126, 127, 190, 191, 599):
        v, v2 = _vis(t), _vis2(t)
        if v2 == 0:
            assert np.all(sh[t] == 0)
        else:
            np.testing.assert_allclose(sh[t, :v], 3.0 / v2, rtol=1e-5)
            assert np.all(sh[t, v:] == 0)


def test_lse_approx_against_plain_loops(oracle):
    """Eq. 7 and Alg. 1 written out with Python loops from the raw keys on a tiny case."""
    p = oracle.Params(lse_mode=1, softmax_scale=0.5)
    rng = np.random.default_rng(2)
    n, G, d = 330, 2, 4
    K = rng.standard_normal((n, d))
    Q = rng.standard_normal((n, G, d))
    Kf, Qf = K.astype(np.float32), Q.astype(np.float32)
    pos = np.array([100, 127, 200, 329], dtype=np.int32)
    sh = oracle.block_scores(Qf[pos], pos, oracle.compress_k(Kf, p), p, oracle.compress_k(Kf, p, level=2))
    K64, Q64 = Kf.astype(np.float64), Qf.astype(np.float64)
    for r, t in enumerate(pos):
        fine = [K64[16 * i:16 * i + 32].mean(0) for i in range(n) if 16 * i + 31 <= t]
        coarse = [K64[64 * i:64 * i + 128].mean(0) for i in range(n) if 64 * i + 127 <= t]
        want = np.zeros(len(fine))
        if coarse:
            for g in range(G):
                lse = math.log(sum(math.exp(0.5 * float(Q64[t, g] @ c)) for c in coarse))
                want += np.array([math.exp(0.5 * float(Q64[t, g] @ f) - lse) for f in fine])
        np.testing.assert_allclose(sh[r, :len(fine)], want, rtol=2e-6, atol=1e-9)
        assert np.all(sh[r, len(fine):] == 0)


def test_lse_approx_rescales_each_head_of_the_exact_scores(oracle):
    """Per head the approximation multiplies the exact softmax row by exp(lse_C1 - lse_C2): with G = 1 the
    ranking of the keys, and therefore the selection, is the exact one."""
    w = _small(n=900, hq=4, hkv=2, d=16, seed=11)
    pe = oracle.Params(n_init=1, n_local=2, topk_total=6, softmax_scale=0.4)
    pa = oracle.Params(n_init=1, n_local=2, topk_total=6, softmax_scale=0.4, lse_mode=1)
    pos = np.arange(127, 900, dtype=np.int32)
    K = w["k"][0]
    kc, kc2 = oracle.compress_k(K, pe), oracle.compress_k(K, pa, level=2)
    Q1 = w["q"][pos, :1]
    se = oracle.block_scores(Q1, pos, kc, pe).astype(np.float64)
    sa = oracle.block_scores(Q1, pos, kc, pa, kc2).astype(np.float64)
    ratio = sa[:, :1] / se[:, :1]
    np.testing.assert_allclose(sa, se * ratio, rtol=2e-5, atol=1e-12)
    # the factor is exp(lse_C1 - lse_C2), computed here with torch from the logits
    for r in (0, 300, len(pos) - 1):
        t = int(pos[r])
        q = torch.from_numpy(Q1[r, 0]).double()
        l1 = torch.logsumexp(0.4 * torch.from_numpy(kc[:_vis(t)]).double() @ q, 0)
        l2 = torch.logsumexp(0.4 * torch.from_numpy(kc2[:_vis2(t)]).double() @ q, 0)
        np.testing.assert_allclose(ratio[r, 0], math.exp(float(l1 - l2)), rtol=1e-5)
    np.testing.assert_array_equal(oracle.topk_blocks(sa.astype(np.float32), pos, pa),
                                  oracle.topk_blocks(se.astype(np.float32), pos, pe))


# ----------------------------------------------------------------------------- stage 3 (Eq. 2, 6)
def test_pool_topk_hand_worked_fixture(oracle):
    g, _ = _read_gold("pool_topk_case.txt")
    shared = np.array(g["shared"], dtype=np.float32)[None, :]
    pos = np.array([447], dtype=np.int32)
    for total in (5, 4, 6):
        p = oracle.Params(n_init=1, n_local=2, topk_total=total)
        idx, cmp = oracle.topk_blocks(shared, pos, p, return_cmp=True)
        np.testing.assert_array_equal(cmp[0], np.array(g["cmp"], dtype=np.float32))
        np.testing.assert_array_equal(idx[0], np.array(g[f"idx_total{total}"], dtype=np.int32))


def _brute_select(row, t, p):
    """Independent restatement with numpy: full stable sort of the remaining blocks."""
    bt = t // p.block_size
    v = _vis(t, p.cmp_len, p.cmp_stride)
    cmp = np.zeros(bt + 1)
    for j in range(bt + 1):
        lo = p.pool_stride * j - p.pool_pad
        w = [row[i] for i in range(lo, lo + p.pool_len) if 0 <= i < v]
        cmp[j] = max(w) if w else 0.0
    forced = set(range(min(p.n_init, bt + 1))) | {j for j in range(bt - p.n_local + 1, bt + 1) if j >= 0}
    rest = [j for j in range(bt + 1) if j not in forced]
    order = sorted(rest, key=lambda j: (-cmp[j], j))
    take = order[:max(0, p.topk_total - p.n_init - p.n_local)]
    return sorted(forced | set(take)), cmp


@pytest.mark.parametrize("pad", [0, 1])
@pytest.mark.parametrize("cfg", [(1, 2, 8), (1, 1, 4), (2, 3, 9), (0, 1, 3), (1, 8, 64)])
def test_topk_against_full_sort(oracle, cfg, pad):
    n_init, n_local, total = cfg
    p = oracle.Params(n_init=n_init, n_local=n_local, topk_total=total, pool_pad=pad)
    rng = np.random.default_rng(11)
    n = 1500
    nc = oracle.num_cmp(n, p)
    pos = np.array(sorted(set(rng.integers(0, n, 80).tolist()) | {0, 30, 31, 63, 64, 127, 128, n - 1}), np.int32)
    shared = np.zeros((len(pos), nc), np.float32)
    for r, t in enumerate(pos):
        v = _vis(int(t))
        # coarse grid of values -> many exact ties, exercising the tie rule
        shared[r, :v] = rng.integers(0, 12, v).astype(np.float32) / 8
    idx, cmp = oracle.topk_blocks(shared, pos, p, return_cmp=True)
    for r, t in enumerate(pos):
        want, cmp_want = _brute_select(shared[r], int(t), p)
        got = [j for j in idx[r] if j >= 0]
        assert got == want, (t, got, want)
        np.testing.assert_array_equal(cmp[r, :len(cmp_want)], cmp_want.astype(np.float32))
        # invariants of Eq. 2
        bt = int(t) // 64
        assert got == sorted(set(got)) and got[-1] == bt
        assert all(j in got for j in range(max(0, bt - n_local + 1), bt + 1))
        assert all(j in got for j in range(min(n_init, bt + 1)))
        rest = bt + 1 - len(set(range(min(n_init, bt + 1))) | set(range(max(0, bt - n_local + 1), bt + 1)))
        assert len(got) == (bt + 1 - rest) + min(total - n_init - n_local, rest)
        assert np.all(idx[r, len(got):] == -1)


def test_planted_topic_block_is_selected(oracle):
    """With a strong topic the block the query's topic was copied from must be chosen whenever it is
    not already forced: the scores really do look at the right keys (catches index/sign slips)."""
    hq, hkv, d, n = 4, 1, 64, 2048
    w = synth.make_prefill(n, hq, hkv, d, seed=5, dtype="fp32", topic_std=0.5, topic_gain=4.0)
    p = oracle.Params(n_init=1, n_local=2, topk_total=8, softmax_scale=d ** -0.5)
    pos = np.arange(n, dtype=np.int32)
    idx = oracle.select_blocks(w["q"], pos, w["k"][0], p)
    src = w["src"][0][0]
    hits = total = 0
    for t in range(256, n):
        total += 1
        hits += int(src[t // 64] in idx[t])
    assert hits == total


# ----------------------------------------------------------------------------- stage 4 (Alg. 2), dense (Eq. 1)
def _masked_dense(q, K, V, mask, scale):
    """Textbook attention with an explicit boolean mask, torch float64.  q [R,G,d], mask [R,n]."""
    q, K, V = (torch.from_numpy(np.asarray(a)).double() for a in (q, K, V))
    z = scale * torch.einsum("rgd,nd->rgn", q, K)
    z = z.masked_fill(~torch.from_numpy(mask)[:, None, :], float("-inf"))
    P = torch.softmax(z, dim=-1)
    return torch.einsum("rgn,nd->rgd", P, V).numpy(), torch.logsumexp(z, dim=-1).numpy()


def test_sparse_attention_equals_bruteforce_masked_dense(oracle):
    w = _small(n=333, hq=4, hkv=2, d=16, seed=21)
    p = oracle.Params(n_init=1, n_local=2, topk_total=4, softmax_scale=0.25, block_size=64)
    n, G = 333, 2
    pos = np.arange(n, dtype=np.int32)
    for h in range(2):
        Qh = w["q"][:, h * G:(h + 1) * G]
        idx = oracle.select_blocks(Qh, pos, w["k"][h], p)
        mask = np.zeros((n, n), dtype=bool)
        for t in range(n):
            for j in idx[t]:
                if j >= 0:
                    mask[t, j * 64:(j + 1) * 64] = True
            mask[t, t + 1:] = False
        assert mask.sum() < np.tril(np.ones((n, n))).sum()        # really sparse
        O, lse = oracle.sparse_attn(Qh, pos, w["k"][h], w["v"][h], idx, p)
        O2, lse2 = _masked_dense(Qh, w["k"][h], w["v"][h], mask, 0.25)
        np.testing.assert_allclose(O, O2, atol=2e-6)
        np.testing.assert_allclose(lse, lse2, atol=2e-6)


def test_sparse_equals_dense_when_every_block_is_kept(oracle):
    w = _small(n=500, hq=4, hkv=1, d=16, seed=22)
    p = oracle.Params(n_init=1, n_local=2, topk_total=8, softmax_scale=0.25)     # nb = 8 <= 8
    pos = np.arange(500, dtype=np.int32)
    idx = oracle.select_blocks(w["q"], pos, w["k"][0], p)
    O, lse = oracle.sparse_attn(w["q"], pos, w["k"][0], w["v"][0], idx, p)
    Od, lsed = oracle.dense_attn(w["q"], pos, w["k"][0], w["v"][0], p)
    np.testing.assert_array_equal(O, Od)
    np.testing.assert_array_equal(lse, lsed)


def test_dense_matches_library_sdpa(oracle):
    w = _small(n=200, hq=6, hkv=2, d=16, seed=23)
    p = oracle.Params(softmax_scale=16 ** -0.5)
    res = oracle.prefill(w["q"], w["k"], w["v"], w["cu_seqlens"], p, force="dense")
    q = torch.from_numpy(w["q"]).double().permute(1, 0, 2)[None]                 # [1,hq,n,d]
    k = torch.from_numpy(w["k"]).double().repeat_interleave(3, dim=0)[None]
    v = torch.from_numpy(w["v"]).double().repeat_interleave(3, dim=0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)[0].permute(1, 0, 2)
    np.testing.assert_allclose(res["out"], ref.numpy(), atol=2e-6)


def test_attention_closed_forms(oracle):
    n, G, d = 300, 2, 8
    p = oracle.Params(n_init=1, n_local=1, topk_total=3, softmax_scale=1.0)
    rng = np.random.default_rng(1)
    K = rng.standard_normal((n, d)).astype(np.float32)
    V = rng.standard_normal((n, d)).astype(np.float32)
    Q = rng.standard_normal((n, G, d)).astype(np.float32)
    pos = np.arange(n, dtype=np.int32)
    idx = oracle.select_blocks(Q, pos, K, p)
    # constant V -> constant output
    O, _ = oracle.sparse_attn(Q, pos, K, np.full_like(V, 1.25), idx, p)
    np.testing.assert_allclose(O, 1.25, atol=1e-6)
    # zero query -> uniform weights: mean of the visible V rows, lse = ln |U|
    O, lse = oracle.sparse_attn(np.zeros_like(Q), pos, K, V, idx, p)
    for t in (0, 63, 64, 200, 299):
        keys = [u for j in idx[t] if j >= 0 for u in range(j * 64, min((j + 1) * 64, t + 1))]
        np.testing.assert_allclose(O[t, 0], V[keys].astype(np.float64).mean(0), atol=1e-6)
        assert abs(lse[t, 1] - math.log(len(keys))) < 1e-6
    # lse really is log sum exp of the scaled logits over the visible set
    O, lse = oracle.sparse_attn(Q, pos, K, V, idx, p)
    t = 277
    keys = [u for j in idx[t] if j >= 0 for u in range(j * 64, min((j + 1) * 64, t + 1))]
    z = Q[t, 1].astype(np.float64) @ K[keys].astype(np.float64).T
    assert abs(lse[t, 1] - np.log(np.exp(z).sum())) < 1e-5


def _selection_mask(idx, n):
    mask = np.zeros((n, n), dtype=bool)
    for t in range(n):
        for j in idx[t]:
            if j >= 0:
                mask[t, j * 64:(j + 1) * 64] = True
        mask[t, t + 1:] = False
    return mask


def test_attention_gradients_match_library_autograd(oracle):
    """The backward formulas against automatic differentiation (a library routine) of textbook masked softmax
    attention in float64: sparse selection and dense, GQA group of 3, loss = <O, dO>."""
    w = _small(n=200, hq=6, hkv=2, d=16, seed=41)
    p = oracle.Params(n_init=1, n_local=1, topk_total=2, softmax_scale=0.3)
    n, G = 200, 3
    pos = np.arange(n, dtype=np.int32)
    rng = np.random.default_rng(5)
    for h in range(2):
        Qh, Kh, Vh = w["q"][:, h * G:(h + 1) * G], w["k"][h], w["v"][h]
        dO = rng.standard_normal(Qh.shape).astype(np.float32)
        idx = oracle.select_blocks(Qh, pos, Kh, p)
        for sel in (idx, None):
            mask = _selection_mask(idx, n) if sel is not None else np.tril(np.ones((n, n), dtype=bool))
            q = torch.from_numpy(Qh).double().requires_grad_()
            k = torch.from_numpy(Kh).double().requires_grad_()
            v = torch.from_numpy(Vh).double().requires_grad_()
            z = torch.einsum("tgd,ud->gtu", q, k) * 0.3
            z = z.masked_fill(~torch.from_numpy(mask)[None], float("-inf"))
            o = torch.einsum("gtu,ud->tgd", torch.softmax(z, dim=-1), v)
            (o * torch.from_numpy(dO).double()).sum().backward()
            dQ, dK, dV = oracle.attn_bwd(Qh, pos, Kh, Vh, sel, dO, p)
            np.testing.assert_allclose(dQ, q.grad.numpy(), atol=1e-12)
            np.testing.assert_allclose(dK, k.grad.numpy(), atol=1e-12)
            np.testing.assert_allclose(dV, v.grad.numpy(), atol=1e-12)


def test_attention_gradients_match_finite_differences_and_invariants(oracle):
    """Central differences of the oracle's own forward on sampled coordinates, and what the mathematics fixes:
    softmax rows sum to 1 => the columns of dV sum to the columns of dO; a constant V => O does not depend on Q or K;
    rows that are not given contribute nothing."""
    w = _small(n=150, hq=2, hkv=1, d=8, seed=42)
    p = oracle.Params(n_init=1, n_local=1, topk_total=2, softmax_scale=0.5)
    n = 150
    pos = np.arange(n, dtype=np.int32)
    Q, K, V = w["q"].astype(np.float64), w["k"][0].astype(np.float64), w["v"][0].astype(np.float64)
    idx = oracle.select_blocks(w["q"], pos, w["k"][0], p)
    mask = _selection_mask(idx, n)
    rng = np.random.default_rng(6)
    dO = rng.standard_normal(Q.shape).astype(np.float32)

    def loss(Q_, K_, V_):
        z = np.einsum("tgd,ud->gtu", Q_, K_) * 0.5
        z = np.where(mask[None], z, -np.inf)
        pr = np.exp(z - z.max(-1, keepdims=True))
        pr /= pr.sum(-1, keepdims=True)
        return float((np.einsum("gtu,ud->tgd", pr, V_) * dO).sum())

    dQ, dK, dV = oracle.attn_bwd(w["q"], pos, w["k"][0], w["v"][0], idx, dO, p)
    h = 1e-5
    for arr, grad, which in ((Q, dQ, 0), (K, dK, 1), (V, dV, 2)):
        for _ in range(12):
            i = tuple(rng.integers(0, s) for s in arr.shape)
            args = [Q.copy(), K.copy(), V.copy()]
            args[which][i] += h
            up = loss(*args)
            args[which][i] -= 2 * h
            fd = (up - loss(*args)) / (2 * h)
            assert abs(fd - grad[i]) < 1e-6 * max(1.0, abs(fd)), (which, i, fd, grad[i])
    np.testing.assert_allclose(dV.sum(0), dO.astype(np.float64).sum((0, 1)), atol=1e-10)
    dQc, dKc, _ = oracle.attn_bwd(w["q"], pos, w["k"][0], np.full_like(w["v"][0], 0.7), idx, dO, p)
    assert np.abs(dQc).max() < 1e-12 and np.abs(dKc).max() < 1e-12
    # a subset of rows: gradients add up over disjoint row sets
    a, b = np.arange(0, 70), np.arange(70, n)
    parts = [oracle.attn_bwd(w["q"][r], pos[r], w["k"][0], w["v"][0], idx[r], dO[r], p) for r in (a, b)]
    np.testing.assert_allclose(parts[0][1] + parts[1][1], dK, atol=1e-12)
    np.testing.assert_allclose(np.concatenate([parts[0][0], parts[1][0]]), dQ, atol=1e-12)


def test_softmax_scale_reaches_both_stages(oracle):
    """A dropped or doubled scale in either stage changes these numbers (d=16: scale 0.25 vs 1)."""
    w = _small(n=200, hq=2, hkv=1, d=16, seed=30)
    pos = np.array([199], dtype=np.int32)
    q = w["q"][pos]
    kc_t = torch.from_numpy(w["k"][0]).double().unfold(0, 32, 16).mean(-1)
    for scale in (0.25, 1.0):
        p = oracle.Params(softmax_scale=scale, n_init=1, n_local=1, topk_total=2)
        sh = oracle.block_scores(q, pos, oracle.compress_k(w["k"][0], p), p)
        v = _vis(199)
        want = torch.softmax(scale * torch.from_numpy(q[0]).double() @ kc_t[:v].T, -1).sum(0).numpy()
        np.testing.assert_allclose(sh[0, :v], want, rtol=2e-6)


# ----------------------------------------------------------------------------- decode, switch, varlen
def test_decode_is_last_prefill_row(oracle):
    hq, hkv, d = 4, 2, 16
    p = oracle.Params(n_init=1, n_local=2, topk_total=5, softmax_scale=0.25)
    for L in (700, 641, 64, 33, 20):          # partial last block, exactly one block, tiny
        w = synth.make_prefill(L, hq, hkv, d, seed=40 + L, dtype="fp32")
        full = oracle.prefill(w["q"], w["k"], w["v"], w["cu_seqlens"], p, rows=[L - 1])
        kc = np.zeros((1, hkv, 704, d), np.float32)
        vc = np.zeros((1, hkv, 704, d), np.float32)
        kc[0, :, :L] = w["k"]
        vc[0, :, :L] = w["v"]
        kc[0, :, L:] = 99.0                    # garbage beyond the context must not matter
        dec = oracle.decode(w["q"][L - 1:L], kc, vc, [L], p)
        np.testing.assert_array_equal(dec["out"][0], full["out"][0])
        np.testing.assert_array_equal(dec["lse"][0], full["lse"][0])
        np.testing.assert_array_equal(dec["idx"][0], full["idx"][:, 0])


def test_varlen_equals_each_sequence_alone_and_switch(oracle):
    hq, hkv, d = 4, 2, 16
    lens = [100, 520, 64, 300]
    p = oracle.Params(n_init=1, n_local=2, topk_total=4, softmax_scale=0.25, dense_threshold=300)
    w = synth.make_varlen(lens, hq, hkv, d, seed=50, dtype="fp32")
    res = oracle.prefill(w["q"], w["k"], w["v"], w["cu_seqlens"], p)
    cu = w["cu_seqlens"]
    for s, n in enumerate(lens):
        a, b = cu[s], cu[s + 1]
        alone = oracle.prefill(w["q"][a:b], w["k"][:, a:b], w["v"][:, a:b], [0, n], p)
        np.testing.assert_array_equal(res["out"][a:b], alone["out"])
        np.testing.assert_array_equal(res["idx"][:, a:b], alone["idx"])
        if n < 300:     # dense side of the switch: no selection, equals Eq. 1
            assert np.all(alone["idx"] == -1)
            dn = oracle.prefill(w["q"][a:b], w["k"][:, a:b], w["v"][:, a:b], [0, n], p, force="dense")
            np.testing.assert_array_equal(alone["out"], dn["out"])
        else:           # n == 300 is NOT below the threshold -> sparse
            assert np.all(alone["idx"][:, -1, 0] == 0)
    # a sequence whose blocks all fit in |I| gives the same result on either side of the switch
    a, b = cu[0], cu[1]
    sp = oracle.prefill(w["q"][a:b], w["k"][:, a:b], w["v"][:, a:b], [0, 100], p, force="sparse")
    np.testing.assert_array_equal(sp["out"], res["out"][a:b])


def test_generator_is_seeded_and_bf16_exact():
    a = synth.make_prefill(256, 4, 2, 16, seed=1, dtype="bf16")
    b = synth.make_prefill(256, 4, 2, 16, seed=1, dtype="bf16")
    c = synth.make_prefill(256, 4, 2, 16, seed=2, dtype="bf16")
    np.testing.assert_array_equal(a["q"], b["q"])
    assert not np.array_equal(a["q"], c["q"])
    for key in ("q", "k", "v"):
        np.testing.assert_array_equal(a[key], synth.round_to_bf16(a[key]))
        t = torch.from_numpy(a[key])
        np.testing.assert_array_equal(t.bfloat16().float().numpy(), a[key])
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    np.testing.assert_array_equal(synth.round_to_bf16(x), torch.from_numpy(x).bfloat16().float().numpy())
