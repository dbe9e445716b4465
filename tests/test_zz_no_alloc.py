"""The entry point that allocates nothing (infllmv2_sparse_decode_static: scratch in a fixed array of the library's
device image) against infllmv2_sparse_decode with a caller workspace: same kernels, so the results must be bit
identical -- on two calls in a row, the second with a smaller input (the array keeps the first call's contents)."""
import ctypes

import numpy as np
import pytest
import torch

import synth
from helpers import to_dev

pytestmark = pytest.mark.gpu


def _caches(m, ctx, seed, lmax):
    w = synth.make_decode(ctx, 32, 2, 128, seed=seed, dtype="bf16", max_len=lmax)
    gp = m.Params.make("bf16", 32, 2, 128, n_init=1, n_local=2, topk_total=8)
    q, kc_, vc_ = to_dev(w["q"], "bf16"), to_dev(w["k_cache"], "bf16"), to_dev(w["v_cache"], "bf16")
    kcc = torch.zeros((len(ctx), 2, max(m.num_cmp(gp, lmax), 1), 128), dtype=torch.float32, device="cuda")
    for b, L in enumerate(ctx):
        if m.num_cmp(gp, L):
            kcb, _ = m.compress_k(gp, kc_[b, :, :L], [0, L])
            kcc[b, :, :kcb.shape[1]] = kcb
    return gp, q, kc_, vc_, kcc


def test_decode_without_allocation_matches_decode_with_workspace():
    import paper_2509_24663_amd as m
    m.lib()
    assert torch.cuda.is_available()
    for call, (ctx, seed, lmax) in enumerate((([5000, 641, 64, 2049, 33, 1], 71, 5056), ([700, 129], 72, 704))):
        gp, q, kc_, vc_, kcc = _caches(m, ctx, seed, lmax)                     # the second input is the smaller one
        di = m.DecodeInfo(ctx)
        want = m.sparse_decode(gp, q, kc_, vc_, kcc, di)
        out = torch.full_like(want[0], 7.0)
        lse = torch.full_like(want[1], 7.0)
        idx = torch.full_like(want[2], 7)
        torch.cuda.synchronize()
        free_before = torch.cuda.mem_get_info()[0]
        m.sparse_decode_static(gp, q, kc_, vc_, kcc, di, out, lse, idx)
        torch.cuda.synchronize()
        # (the first call on a GPU may make the driver place the library's device image, array included; from then
        # on the device's free memory must not move)
        if call > 0:
            assert torch.cuda.mem_get_info()[0] == free_before
        assert torch.equal(out, want[0]) and torch.equal(lse, want[1]) and torch.equal(idx, want[2]), ctx
    # a step beyond the fixed array is refused on the host, with the status that says why
    big = m.Params.make("bf16", 32, 2, 128)
    assert m.decode_workspace_bytes(big, 64, 262144) > m.sparse_decode_static_capacity()
    ctxs = np.full(64, 262144, dtype=np.int32)
    one = ctypes.c_void_p(256)
    st = m.lib().infllmv2_sparse_decode_static(ctypes.byref(big), one, one, one, 1 << 26, 1 << 25, 128, one, 1 << 22,
                                               ctxs.ctypes.data_as(ctypes.c_void_p), one, 64, None, one, None, None)
    assert st == -3
