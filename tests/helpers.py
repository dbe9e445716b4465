"""Shared helpers for the GPU parity tests: upload synthetic inputs, compare with the oracle."""
from __future__ import annotations

import numpy as np
import torch

TIE_RTOL = 1e-3          # selection may differ from the oracle only among blocks this close to the threshold
FP32_MAX_ABS = 1e-4      # attention output tolerance, fp32 data
BF16_MAX_ABS = 2e-2      # attention output tolerance, bf16 data
BF16_MEAN_ABS = 2e-3


def to_dev(a: np.ndarray, dtype: str) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)         # values are already bf16-exact
    return t.cuda()


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy() if t.dtype != torch.int32 else t.detach().cpu().numpy()


def out_tolerances(dtype: str):
    return (FP32_MAX_ABS, None) if dtype == "fp32" else (BF16_MAX_ABS, BF16_MEAN_ABS)


SCORE_RTOL = 5e-4        # stage-2 scores: K^{C1} enters the MFMA as fp16 (11-bit significand), see below
TIE_FLIP_RATE_MAX = 0.05  # share of sampled rows whose list may differ from the oracle's by near-ties


def prefill_lse_atol(dtype: str) -> float:
    """Tolerance for the log-sum-exp of the prefill kernels.  The logits are formed from Q and K as stored (the
    power-of-two part of softmax_scale * log2(e) goes into Q exactly, the mantissa multiplies the fp32
    accumulator), accumulated in fp32; what is left is the fast exponential / logarithm (relative 2^-22) and the
    order of a sum over up to 131072 keys: 2e-3 is the bar the bf16 decode path has always met, 1e-4 for fp32
    data (whose logits are accumulated by plain fp32 loops)."""
    return 2e-3 if dtype == "bf16" else 1e-4


def assert_out_close(got: np.ndarray, want: np.ndarray, dtype: str, what: str = "out"):
    diff = np.abs(got.astype(np.float64) - want.astype(np.float64))
    max_abs, mean_abs = out_tolerances(dtype)
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    assert diff.max() <= max_abs, f"{what}: max-abs {diff.max():.3e} > {max_abs}"
    if mean_abs is not None:
        assert diff.mean() <= mean_abs, f"{what}: mean-abs {diff.mean():.3e} > {mean_abs}"
    return float(diff.max()), float(diff.mean())


def check_selection(idx_gpu: np.ndarray, idx_orc: np.ndarray, cmp_orc: np.ndarray, pos: np.ndarray, n_init: int,
                    n_local: int, block: int = 64):
    """Rows must hold the same block sets; a differing block is allowed only if its oracle score is within
    TIE_RTOL (relative) of the oracle's smallest selected top-k score.  Returns (#rows differing, #blocks)."""
    assert idx_gpu.shape == idx_orc.shape
    rows_diff = blocks_diff = 0
    neq = np.nonzero((idx_gpu != idx_orc).any(axis=1))[0]
    for r in neq:
        g = set(int(x) for x in idx_gpu[r] if x >= 0)
        o = set(int(x) for x in idx_orc[r] if x >= 0)
        assert len(g) == len(o), f"row {r}: {len(g)} blocks selected, oracle {len(o)}"
        gl = [x for x in idx_gpu[r] if x >= 0]
        assert gl == sorted(g), f"row {r}: not ascending/unique"
        bt = int(pos[r]) // block
        forced = set(range(min(n_init, bt + 1))) | set(range(max(0, bt - n_local + 1), bt + 1))
        assert forced <= g, f"row {r}: forced blocks missing"
        assert max(g) <= bt
        topk_o = [j for j in o if j not in forced]
        tau = min(float(cmp_orc[r, j]) for j in topk_o)
        for j in g ^ o:
            s = float(cmp_orc[r, j])
            assert abs(s - tau) <= TIE_RTOL * tau + 1e-30, (
                f"row {r} (pos {pos[r]}): block {j} score {s:.6g} vs threshold {tau:.6g} is not a tie")
        rows_diff += 1
        blocks_diff += len(g ^ o) // 2
    return rows_diff, blocks_diff
