"""Parity at the full BASELINE sizes, through the same entry points and launch configuration bench.py times.
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
    print("C2", st)
    assert st["rows"] >= 700


def test_c2_32k_sampled_lse_approximation(m, oracle):
    """The same workload with the LSE Approximation of Sec. 3.4 (lse_mode 1) in stage 2."""
    import dataclasses
    cfg = synth.CONFIGS["C2"]
    w = synth.make_config(cfg)
    rows = _sample_rows(w["cu_seqlens"], np.random.default_rng(12), 4, 192)
    gp = m.Params.from_config(cfg, lse_mode=1)
    op = dataclasses.replace(oracle.Params.from_config(cfg), lse_mode=1)
    st = _run_prefill_case(m, oracle, w, gp, op, "bf16", rows=rows)
    print("C2 lse_mode 1", st)
    assert st["rows"] >= 400


def test_c3_128k_sampled_sparse_and_dense(m, oracle):
    cfg = synth.CONFIGS["C3"]
    w = synth.make_config(cfg)
    gp, op = m.Params.from_config(cfg), oracle.Params.from_config(cfg)
    rows = _sample_rows(w["cu_seqlens"], np.random.default_rng(3), 4, 192)
    st = _run_prefill_case(m, oracle, w, gp, op, "bf16", rows=rows)
    print("C3", st)
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
    rows = _sample_rows(w["cu_seqlens"], np.random.default_rng(5), 2, 48)
    st = _run_prefill_case(m, oracle, w, m.Params.from_config(cfg), oracle.Params.from_config(cfg), "bf16", rows=rows)
    print("C5", st)


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
