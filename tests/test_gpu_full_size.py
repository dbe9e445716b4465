"""Parity at the full sizes of the workloads in synth.CONFIGS, through the same entry points and launch configuration bench.py times.
The oracle cannot afford every row at these sizes, so it is run on a stratified sample of query rows (rows are
independent: parity on a sampled row is exact for that row): whole query blocks (first, last, random) plus
random single tokens, per sequence."""
import numpy as np
import pytest
import torch

import synth
from helpers import assert_out_close, to_dev, to_np
from test_gpu_parity import _check_decode, _run_prefill_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def m():
    import paper_2509_24663_amd as m
    m.lib()
    return m


def _sample_rows(cu, rng, blocks_per_seq, singles_per_seq):
    rows = []
    for s in range(len(cu) - 1):
        a, b = int(cu[s]), int(cu[s + 1])
        n = b - a
        nb = (n + 63) // 64
        pick = {0, nb - 1} | set(rng.integers(0, nb, size=min(blocks_per_seq, nb)).tolist())
        for j in pick:
            rows.extend(range(a + j * 64, min(a + (j + 1) * 64, b)))
        rows.extend((a + rng.integers(0, n, size=min(singles_per_seq, n))).tolist())
    return np.unique(np.asarray(rows, dtype=np.int64))


def test_c2_32k_sampled(m, oracle):
    cfg = synth.CONFIGS["C2"]
    w = synth.make_config(cfg)
    rows = _sample_rows(w["cu_seqlens"], np.random.default_rng(2), 6, 256)
    st = _run_prefill_case(m, oracle, w, m.Params.from_config(cfg), oracle.Params.from_config(cfg), "bf16", rows=rows)
    _report("C2", st)
    assert st["rows"] >= 1400


def test_c2_32k_sampled_lse_approximation(m, oracle):
    """The same workload with the LSE Approximation of Sec. 3.4 (lse_mode 1) in stage 2."""
    import dataclasses
    cfg = synth.CONFIGS["C2"]
    w = synth.make_config(cfg)
    rows = _sample_rows(w["cu_seqlens"], np.random.default_rng(12), 4, 192)
    gp = m.Params.from_config(cfg, lse_mode=1)
    op = dataclasses.replace(oracle.Params.from_config(cfg), lse_mode=1)
    st = _run_prefill_case(m, oracle, w, gp, op, "bf16", rows=rows)
    _report("C2 lse_mode 1", st)
    assert st["rows"] >= 800


def _report(name, st):
    print(f"{name}: {st['rows']} (row, KV head) pairs sampled, {st['rows_diff']} differ from the oracle's lists by near-ties "
          f"({100.0 * st['rows_diff'] / max(st['rows'], 1):.2f} %), largest relative score error {st['score_rel']:.2e}, "
          f"out max-abs {st['max_abs']:.2e}, lse max-abs {st['lse_abs']:.2e}", flush=True)


def test_c3_128k_sampled_sparse_and_dense(m, oracle):
    """Config 3 (the workload bench.py times): 32 random query blocks plus the first and last one, and 2048 random
    single tokens, for both KV heads -- two-stage path; then the fused-pooling path bench.py's step uses, against
    the oracle directly on a second sample."""
    cfg = synth.CONFIGS["C3"]
    w = synth.make_config(cfg)
    gp, op = m.Params.from_config(cfg), oracle.Params.from_config(cfg)
    rows = _sample_rows(w["cu_seqlens"], np.random.default_rng(3), 32, 2048)
    assert len(rows) >= 4000
    st = _run_prefill_case(m, oracle, w, gp, op, "bf16", rows=rows)
    _report("C3 two-stage", st)
    rows = _sample_rows(w["cu_seqlens"], np.random.default_rng(33), 8, 512)
    st = _run_prefill_case(m, oracle, w, gp, op, "bf16", rows=rows, fused_pool=True)
    _report("C3 fused pooling", st)
    # the library's dense path at the same shape, on a smaller sample (a dense oracle row costs ~1e9 flop)
    q, k, v = (to_dev(w[x], "bf16") for x in ("q", "k", "v"))
    out, lse = m.dense_attn_fwd(gp, q, k, v, [0, cfg.seq_len])
    torch.cuda.synchronize()
    drows = np.unique(np.concatenate([[0, 63, 64, 4095, cfg.seq_len - 1],
                                      np.random.default_rng(4).integers(0, cfg.seq_len, 43)]))
    pos = drows.astype(np.int32)
    G = cfg.group
    o_g = to_np(out[torch.from_numpy(drows).cuda()])
    for h in range(cfg.num_kv_heads):
        O, L = oracle.dense_attn(w["q"][drows, h * G:(h + 1) * G], pos, w["k"][h], w["v"][h], op)
        assert_out_close(o_g[:, h * G:(h + 1) * G], O, "bf16", "dense out at 128K")


def test_c5_varlen_mixed_dense_sparse(m, oracle):
    cfg = synth.CONFIGS["C5"]
    w = synth.make_config(cfg)
    assert list(w["cu_seqlens"]) == [0, 512, 2560, 6656, 14848, 31232, 55808, 88576, 154112]
    rows = _sample_rows(w["cu_seqlens"], np.random.default_rng(5), 4, 256)
    st = _run_prefill_case(m, oracle, w, m.Params.from_config(cfg), oracle.Params.from_config(cfg), "bf16", rows=rows)
    _report("C5", st)


def test_paper_budget_96_blocks_at_32k(m, oracle):
    """The paper's own budget (Sec. 4.1): |I| = 96 = 1 initial + 63 top-k + 32 local blocks, end to end at 32K
    tokens, two-stage and fused."""
    import dataclasses
    cfg = synth.CONFIGS["C2"]
    w = synth.make_config(cfg)
    gp = m.Params.from_config(cfg, n_init=1, n_local=32, topk_total=96)
    op = dataclasses.replace(oracle.Params.from_config(cfg), n_init=1, n_local=32, topk_total=96)
    rows = _sample_rows(w["cu_seqlens"], np.random.default_rng(96), 6, 256)
    _report("32K, |I| = 96", _run_prefill_case(m, oracle, w, gp, op, "bf16", rows=rows))
    rows = _sample_rows(w["cu_seqlens"], np.random.default_rng(97), 3, 128)
    _report("32K, |I| = 96, fused", _run_prefill_case(m, oracle, w, gp, op, "bf16", rows=rows, fused_pool=True))


def test_sweep_budget_16_blocks_at_128k(m, oracle):
    """The kernel-speed experiment's budget (Sec. 4.3: 16 selected blocks; here 1 initial + 8 local + 7 top-k) at its
    longest length, 128K tokens, end to end through the fused path the sweep is timed on."""
    import dataclasses
    cfg = synth.CONFIGS["C3"]
    w = synth.make_config(cfg)
    gp = m.Params.from_config(cfg, n_init=1, n_local=8, topk_total=16)
    op = dataclasses.replace(oracle.Params.from_config(cfg), n_init=1, n_local=8, topk_total=16)
    rows = _sample_rows(w["cu_seqlens"], np.random.default_rng(16), 8, 512)
    _report("128K, 16 blocks, fused", _run_prefill_case(m, oracle, w, gp, op, "bf16", rows=rows, fused_pool=True))


def test_c3_with_a_budget_of_136_blocks(m, oracle):
    """At 128K tokens a 16-token tile's union list may then hold more than 2 * 1024 entries, more than one thread per
    interval record can pack, and the tile kernel walks one entry per barrier interval instead of two (the same path
    as for sequences whose block masks leave no room for four LDS stages).  Whole sparse path against the oracle on
    sampled rows."""
    import dataclasses
    cfg = synth.CONFIGS["C3"]
    w = synth.make_config(cfg)
    gp = m.Params.from_config(cfg, n_init=1, n_local=8, topk_total=136)
    op = dataclasses.replace(oracle.Params.from_config(cfg), n_init=1, n_local=8, topk_total=136)
    rows = _sample_rows(w["cu_seqlens"], np.random.default_rng(136), 2, 160)
    _report("128K, 136 blocks", _run_prefill_case(m, oracle, w, gp, op, "bf16", rows=rows, fused_pool=True))


def test_sparse_attention_beyond_384k_tokens(m, oracle):
    """Past about 384K tokens the tile kernel's per-block masks leave no room for four LDS stages, and block lists
    are walked one entry per barrier interval instead of two.  Stage 4 alone on a 400K-token sequence with valid
    random block lists (forced blocks plus random earlier ones), against the oracle on sampled rows."""
    n, hq, hkv, d, K = 400000, 32, 2, 128, 16
    G = hq // hkv
    gen = torch.Generator(device="cuda").manual_seed(4001)
    q = torch.randn((n, hq, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn((hkv, n, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((hkv, n, d), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    gp = m.Params.make("bf16", hq, hkv, d, n_init=1, n_local=2, topk_total=K)
    op = oracle.Params(n_init=1, n_local=2, topk_total=K, softmax_scale=float(gp.softmax_scale))
    # block lists: block 0, the two most recent blocks, and up to 13 distinct random earlier ones, ascending, -1 padded
    t = torch.arange(n, device="cuda")
    bt = (t // 64)[None, :, None]                                               # [1, n, 1]
    cand = (torch.rand((hkv, n, K - 3), generator=gen, device="cuda") * (bt - 1).clamp(min=1)).long() + 1
    cand = torch.where(cand < bt - 1, cand, torch.full_like(cand, -1))          # only blocks in (0, bt - 1)
    forced = torch.cat([torch.zeros_like(bt), bt - 1, bt], dim=2).expand(hkv, n, 3).clone()
    forced[:, :, 1] = torch.where(forced[:, :, 1] > 0, forced[:, :, 1], torch.full_like(forced[:, :, 1], -1))
    forced[:, :, 2] = torch.where(forced[:, :, 2] > 0, forced[:, :, 2], torch.full_like(forced[:, :, 2], -1))
    allb = torch.cat([forced, cand], dim=2)
    big = torch.iinfo(torch.int64).max
    srt, _ = torch.sort(torch.where(allb >= 0, allb, torch.full_like(allb, big)), dim=2)
    dup = torch.zeros_like(srt, dtype=torch.bool)
    dup[:, :, 1:] = srt[:, :, 1:] == srt[:, :, :-1]
    srt = torch.where(dup, torch.full_like(srt, big), srt)
    srt, _ = torch.sort(srt, dim=2)
    idx = torch.where(srt == big, torch.full_like(srt, -1), srt).to(torch.int32).contiguous()
    out, lse = m.sparse_attn_fwd(gp, q, k, v, idx, [0, n])
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 63, 64, 130, n - 1], np.random.default_rng(5).integers(0, n, 91)]))
    rows_d = torch.from_numpy(rows).cuda()
    o_g, l_g, idx_g = to_np(out[rows_d]), to_np(lse[:, rows_d]), to_np(idx[:, rows_d])
    qn = to_np(q[rows_d])
    pos = rows.astype(np.int32)
    for h in range(hkv):
        kh, vh = to_np(k[h]), to_np(v[h])
        O, L = oracle.sparse_attn(qn[:, h * G:(h + 1) * G], pos, kh, vh, idx_g[h], op)
        assert_out_close(o_g[:, h * G:(h + 1) * G], O, "bf16", "out at 400K tokens")
        np.testing.assert_allclose(l_g[h * G:(h + 1) * G].T, L, atol=2e-3)


def test_decode_context_of_400k_tokens(m, oracle):
    """A context near the upper limit of the decode selection kernel (its score row must fit in LDS, ~419K
    tokens), with a much shorter sequence in the same batch; a longer one is refused, not mis-computed."""
    ctx = [400000, 70000]
    w = synth.make_decode(ctx, 32, 2, 128, seed=31, dtype="bf16")
    gp = m.Params.make("bf16", 32, 2, 128, n_init=1, n_local=8, topk_total=64)
    op = oracle.Params(n_init=1, n_local=8, topk_total=64, softmax_scale=float(gp.softmax_scale))
    assert _check_decode(m, oracle, w, ctx, gp, op, "bf16") == 4


def test_c2_32k_backward_sampled(m, oracle):
    """Gradients of stage 4 at config 2's full size.  dQ of a row depends on that row alone, so it is checked on a
    sample of rows; dK / dV of a key block sum over every row that selected the block, so one block is checked
    with the oracle run on exactly those rows (taken from the GPU's selection)."""
    cfg = synth.CONFIGS["C2"]
    w = synth.make_config(cfg)
    gp, op = m.Params.from_config(cfg), oracle.Params.from_config(cfg)
    n, G, hkv = cfg.seq_len, cfg.group, cfg.num_kv_heads
    q, k, v = (to_dev(w[x], "bf16") for x in ("q", "k", "v"))
    rng = np.random.default_rng(77)
    dout_np = synth.round_to_bf16(rng.standard_normal(w["q"].shape).astype(np.float32))
    dout = to_dev(dout_np, "bf16")
    res = m.sparse_prefill(gp, q, k, v, [0, n], fused_pool=True)
    dq, dk, dv = m.sparse_attn_bwd(gp, q, k, v, res["block_idx"], res["out"], res["lse"], dout, [0, n])
    torch.cuda.synchronize()
    idx_g = to_np(res["block_idx"])
    print("C2 backward: GPU done, oracle on sampled rows and one key block ...", flush=True)

    def rel(got, ref):
        scale = max(float(np.abs(ref).max()), 0.1)
        err = np.abs(got.astype(np.float64) - ref) / scale
        return float(err.max()), float(err.mean())

    rows = np.unique(np.concatenate([[0, 63, 64, n - 1], rng.integers(0, n, 28)])).astype(np.int32)
    dq_g = to_np(dq[torch.from_numpy(rows.astype(np.int64)).cuda()])
    h = 1
    dQ, _, _ = oracle.attn_bwd(w["q"][rows, h * G:(h + 1) * G], rows, w["k"][h], w["v"][h], idx_g[h, rows],
                               dout_np[rows, h * G:(h + 1) * G], op)
    mx, mean = rel(dq_g[:, h * G:(h + 1) * G], dQ)
    assert mx <= 2e-2 and mean <= 2e-3, ("dq", mx, mean)
    dk_g, dv_g = to_np(dk[h]), to_np(dv[h])
    for j in (401,):                                       # a block outside the forced ranges of most rows
        users = np.nonzero((idx_g[h] == j).any(-1))[0].astype(np.int32)
        assert 64 < len(users) < 6000
        _, dK, dV = oracle.attn_bwd(w["q"][users, h * G:(h + 1) * G], users, w["k"][h], w["v"][h], idx_g[h, users],
                                    dout_np[users, h * G:(h + 1) * G], op)
        for name, got, ref in (("dk", dk_g, dK), ("dv", dv_g, dV)):
            mx, mean = rel(got[j * 64:(j + 1) * 64], ref[j * 64:(j + 1) * 64])
            assert mx <= 2e-2 and mean <= 2e-3, (name, j, len(users), mx, mean)
