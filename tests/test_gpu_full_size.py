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
