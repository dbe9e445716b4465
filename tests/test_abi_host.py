"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def m():
    import paper_2509_24663_amd as m
    if not os.path.exists(os.path.join(ROOT, "paper_2509_24663_amd", "libinfllmv2.so")):
        from paper_2509_24663_amd import build
        build.build(force=False)
    return m


def test_header_symbols_are_exported(m):
    hdr = open(os.path.join(ROOT, "include", "infllmv2.h")).read()
    declared = set(re.findall(r"\b(infllmv2_[a-z_0-9]+)\s*\(", hdr))
    assert {"infllmv2_compress_k", "infllmv2_block_scores", "infllmv2_topk_blocks", "infllmv2_sparse_attn_fwd",
            "infllmv2_sparse_decode", "infllmv2_dense_attn_fwd"} <= declared
    L = m.lib()
    for name in declared:
        assert hasattr(L, name), f"{name} declared in the header but not exported"
    from paper_2509_24663_amd import binding
    assert set(binding.exported_symbols()) == declared


def test_struct_layout_matches_header(m):
    hdr = open(os.path.join(ROOT, "include", "infllmv2.h")).read()
    body = re.search(r"typedef struct infllmv2_params \{(.*?)\} infllmv2_params;", hdr, re.S).group(1)
    fields = re.findall(r"^\s*(?:int32_t|float)\s+([a-z_]+);", body, re.M)
    assert fields == [f[0] for f in m.Params._fields_]
    assert ctypes.sizeof(m.Params) == 4 * len(fields)


def test_num_cmp_and_strings(m):
    p = m.Params.make("bf16", 32, 2, 128)
    assert [m.num_cmp(p, n) for n in (0, 31, 32, 47, 48, 2048, 32768, 131072)] == [0, 0, 1, 1, 2, 127, 2047, 8191]
    assert m.status_string(0) == "ok"
    assert "workspace" in m.status_string(-3)
    assert m.version().startswith("infllmv2")


def _call_compress(m, p, cu, total_c=100, k=1, kc=1, cuc=1, tok=256, head=128):
    cu = np.asarray(cu, dtype=np.int32)
    return m.lib().infllmv2_compress_k(ctypes.byref(p), ctypes.c_void_p(k), tok, head,
                                       cu.ctypes.data_as(ctypes.c_void_p), ctypes.c_void_p(1), len(cu) - 1,
                                       ctypes.c_void_p(kc), ctypes.c_void_p(cuc), total_c, None)


def test_validation_errors_before_launch(m):
    good = dict(dtype="bf16", num_q_heads=32, num_kv_heads=2, head_dim=128)
    INVALID, UNSUPPORTED = -1, -2
    cases = [
        (dict(good, num_q_heads=31), INVALID),            # hq % hkv != 0
        (dict(good, head_dim=96), UNSUPPORTED),
        (dict(good, num_q_heads=64), UNSUPPORTED),        # G = 32 > 16
    ]
    for kw, want in cases:
        p = m.Params.make(kw.pop("dtype"), kw.pop("num_q_heads"), kw.pop("num_kv_heads"), kw.pop("head_dim"))
        assert _call_compress(m, p, [0, 64]) == want
    for over, want in [(dict(n_local=0), INVALID), (dict(n_init=60, n_local=8, topk_total=64), INVALID),
                       (dict(block_size=128), UNSUPPORTED), (dict(cmp_stride=0), INVALID),
                       (dict(cmp_len=8, cmp_stride=16), INVALID), (dict(lse_mode=2), INVALID), (dict(lse_mode=1, cmp_len=24), UNSUPPORTED),
                       (dict(softmax_scale=0.0), INVALID), (dict(topk_total=2048), UNSUPPORTED)]:
        p = m.Params.make("bf16", 32, 2, 128, **over)
        assert _call_compress(m, p, [0, 64]) == want, over
    p = m.Params.make("bf16", 32, 2, 128)
    assert _call_compress(m, p, [1, 64]) == INVALID                 # cu[0] != 0
    assert _call_compress(m, p, [0, 64, 32]) == INVALID             # decreasing
    assert _call_compress(m, p, [0, 64], k=0) == INVALID            # null K
    assert _call_compress(m, p, [0, 64], total_c=2) == INVALID      # kc too small: nc(64) = 3
    assert _call_compress(m, p, [0, 64], tok=64) == INVALID         # token stride < head_dim
    assert m.lib().infllmv2_compress_k(None, None, 0, 0, None, None, 0, None, None, 0, None) == INVALID
    # cache append: shrinking lengths and a compressed-key plane that is too small are caught on the host;
    # a step that completes no window returns before touching any pointer
    L = m.lib()
    def _app(prev, ctx, kc_stride):
        pv, cx = np.array(prev, np.int32), np.array(ctx, np.int32)
        return L.infllmv2_compress_k_append(ctypes.byref(p), ctypes.c_void_p(256), 1 << 20, 1 << 16, 128,
                                            ctypes.c_void_p(256), kc_stride, pv.ctypes.data_as(ctypes.c_void_p),
                                            ctypes.c_void_p(256), cx.ctypes.data_as(ctypes.c_void_p),
                                            ctypes.c_void_p(256), len(prev), None)
    assert _app([100], [90], 1 << 16) == INVALID
    assert _app([0], [64], 2 * 128) == INVALID                       # nc(64) = 3 rows needed
    assert _app([33], [47], 0) == 0                                  # no window completed: nothing to do
    # decode: workspace size query and too-small workspace
    need = m.decode_workspace_bytes(p, 16, 65536)
    assert need > 16 * 2 * 4095 * 4
    ctx = np.array([100, 200], dtype=np.int32)
    st = m.lib().infllmv2_sparse_decode(ctypes.byref(p), ctypes.c_void_p(256), ctypes.c_void_p(256),
                                        ctypes.c_void_p(256), 1 << 20, 1 << 16, 128, ctypes.c_void_p(256), 1 << 16,
                                        ctx.ctypes.data_as(ctypes.c_void_p), ctypes.c_void_p(256), 2, None,
                                        ctypes.c_void_p(256), None, ctypes.c_void_p(256), 16, None)
    assert st == -3
    ctx[1] = 0
    st = m.lib().infllmv2_sparse_decode(ctypes.byref(p), ctypes.c_void_p(256), ctypes.c_void_p(256),
                                        ctypes.c_void_p(256), 1 << 20, 1 << 16, 128, ctypes.c_void_p(256), 1 << 16,
                                        ctx.ctypes.data_as(ctypes.c_void_p), ctypes.c_void_p(256), 2, None,
                                        ctypes.c_void_p(256), None, ctypes.c_void_p(256), 1 << 30, None)
    assert st == INVALID


def test_pooled_entry_points_validate_on_the_host(m):
    """The fused-pooling forms of stages 2 and 3: row stride counted in selection blocks, null pointers,
    empty batches -- all decided before anything is launched."""
    INVALID = -1
    L = m.lib()
    p = m.Params.make("bf16", 32, 2, 128)
    cu = np.array([0, 1000], dtype=np.int32)                         # 16 blocks
    cu_p, one = cu.ctypes.data_as(ctypes.c_void_p), ctypes.c_void_p(256)
    big = 1 << 30
    assert L.infllmv2_block_scores_pooled(ctypes.byref(p), one, one, 61, cu_p, one, one, 1, one, 15, one, big, None) == INVALID
    assert L.infllmv2_block_scores_pooled(ctypes.byref(p), None, one, 61, cu_p, one, one, 1, one, 16, one, big, None) == INVALID
    assert L.infllmv2_block_scores_pooled(ctypes.byref(p), one, one, 61, cu_p, one, one, 1, None, 16, one, big, None) == INVALID
    assert L.infllmv2_topk_pooled(ctypes.byref(p), one, 15, cu_p, one, 1, one, None) == INVALID
    assert L.infllmv2_topk_pooled(ctypes.byref(p), None, 16, cu_p, one, 1, one, None) == INVALID
    empty = np.array([0, 0], dtype=np.int32).ctypes.data_as(ctypes.c_void_p)
    assert L.infllmv2_block_scores_pooled(ctypes.byref(p), None, None, 0, empty, one, None, 1, None, 0, None, 0, None) == 0
    assert L.infllmv2_topk_pooled(ctypes.byref(p), None, 0, empty, one, 1, None, None) == 0
    bad = m.Params.make("bf16", 32, 2, 128, pool_stride=0)
    assert L.infllmv2_block_scores_pooled(ctypes.byref(bad), one, one, 61, cu_p, one, one, 1, one, 16, one, big, None) == INVALID


def test_backward_entry_point_validates_on_the_host(m):
    INVALID, TOO_SMALL = -1, -3
    L = m.lib()
    p = m.Params.make("bf16", 32, 2, 128)
    cu = np.array([0, 100], dtype=np.int32)
    cu_p, one = cu.ctypes.data_as(ctypes.c_void_p), ctypes.c_void_p(256)

    def call(**over):
        a = dict(q=one, k=one, v=one, ts=256, hs=128, idx=one, out=one, lse=one, dout=one, dq=one, dk=one, dv=one,
                 ws=one, ws_bytes=1 << 30)
        a.update(over)
        return L.infllmv2_sparse_attn_bwd(ctypes.byref(p), a["q"], a["k"], a["v"], a["ts"], a["hs"], a["idx"], a["out"],
                                          a["lse"], a["dout"], cu_p, one, 1, a["dq"], a["dk"], a["dv"], a["ws"],
                                          a["ws_bytes"], None)
    for name in ("q", "k", "v", "out", "lse", "dout", "dq", "dk", "dv"):
        assert call(**{name: None}) == INVALID, name
    assert call(ts=64) == INVALID                                    # token stride < head_dim
    assert call(dk=ctypes.c_void_p(260)) == INVALID                  # dK not 16-byte aligned
    need = m.workspace_bytes(m.OP_SPARSE_ATTN_BWD_MIN, p, 1, 100, 100)
    assert need > 0 and m.workspace_bytes(m.OP_SPARSE_ATTN_BWD, p, 1, 100, 100) > need
    assert call(ws=None) == INVALID and call(ws=ctypes.c_void_p(264)) == INVALID      # scratch missing / misaligned
    assert call(ws_bytes=need - 256) == TOO_SMALL
    empty = np.array([0, 0], dtype=np.int32).ctypes.data_as(ctypes.c_void_p)
    assert L.infllmv2_sparse_attn_bwd(ctypes.byref(p), None, None, None, 0, 0, None, None, None, None, empty, one, 1,
                                      None, None, None, None, 0, None) == 0


def test_workspace_query_and_too_small_workspaces(m):
    """Every call that keeps something between its kernels takes caller-owned scratch: the size query bounds the
    exact need of any batch with those totals, and a workspace that is missing, misaligned or one byte-block short
    is rejected before anything is launched (the pointers here are not device memory)."""
    INVALID, TOO_SMALL = -1, -3
    L = m.lib()
    p = m.Params.make("bf16", 32, 2, 128, topk_total=16)
    cu = np.array([0, 1000, 1000, 5000], dtype=np.int32)            # 16 + 0 + 63 blocks; nc = 61 + 0 + 249
    cu_p, one = cu.ctypes.data_as(ctypes.c_void_p), ctypes.c_void_p(256)
    batch, total, mx = 3, 5000, 4000
    # exact needs, from the layouts the kernels use
    blocks = 16 + 63
    kt = (61 + 63) // 64 + (249 + 63) // 64
    exact_attn = blocks * 2 * 128 * 64 * 2
    exact_scores = -(-(2 * kt * (64 * 128 * 2 + 4)) // 256) * 256
    q_attn = m.workspace_bytes(m.OP_SPARSE_ATTN_FWD, p, batch, total, mx)
    q_scores = m.workspace_bytes(m.OP_BLOCK_SCORES, p, batch, total, mx)
    assert exact_attn <= q_attn <= exact_attn + 3 * 2 * 16384
    assert exact_scores <= q_scores <= exact_scores + 4 * 2 * 16640
    assert m.workspace_bytes(m.OP_DENSE_ATTN_FWD, p, batch, total, mx) == q_attn
    assert m.workspace_bytes(m.OP_BLOCK_SCORES_POOLED, p, batch, total, mx) == q_scores
    lse1 = m.Params.make("bf16", 32, 2, 128, lse_mode=1)
    assert m.workspace_bytes(m.OP_BLOCK_SCORES, lse1, batch, total, mx) > q_scores      # coarse key tiles too
    for op in (m.OP_COMPRESS_K, m.OP_TOPK_BLOCKS, m.OP_TOPK_POOLED, m.OP_COMPRESS_K_APPEND, 99):
        assert m.workspace_bytes(op, p, batch, total, mx) == 0
    assert m.workspace_bytes(m.OP_SPARSE_DECODE, p, 16, 0, 65536) == m.decode_workspace_bytes(p, 16, 65536)
    # shapes served by the plain kernels keep nothing between launches in the forward direction
    small = m.Params.make("fp32", 4, 1, 64, topk_total=8, n_local=2)
    assert m.workspace_bytes(m.OP_SPARSE_ATTN_FWD, small, 1, 2048, 2048) == 0
    assert m.workspace_bytes(m.OP_BLOCK_SCORES, small, 1, 2048, 2048) == 0
    assert m.workspace_bytes(m.OP_SPARSE_ATTN_BWD, small, 1, 2048, 2048) == 2048 * 4 * 4
    bad = m.Params.make("bf16", 32, 2, 96)
    assert m.workspace_bytes(m.OP_SPARSE_ATTN_FWD, bad, 1, 100, 100) == 0               # rejected parameters

    def attn(sparse, ws, nbytes):
        if sparse:
            return L.infllmv2_sparse_attn_fwd(ctypes.byref(p), one, one, one, 128, 1 << 20, one, cu_p, one, batch, one,
                                              one, ws, nbytes, None)
        return L.infllmv2_dense_attn_fwd(ctypes.byref(p), one, one, one, 128, 1 << 20, cu_p, one, batch, one, one, ws,
                                         nbytes, None)

    def scores(pooled, ws, nbytes):
        fn = L.infllmv2_block_scores_pooled if pooled else L.infllmv2_block_scores
        return fn(ctypes.byref(p), one, one, 400, cu_p, one, one, batch, one, 252 if not pooled else 63, ws, nbytes, None)

    for sparse in (True, False):
        assert attn(sparse, None, 1 << 30) == INVALID
        assert attn(sparse, ctypes.c_void_p(256 + 64), 1 << 30) == INVALID
        assert attn(sparse, one, exact_attn - 256) == TOO_SMALL
    for pooled in (True, False):
        assert scores(pooled, None, 1 << 30) == INVALID
        assert scores(pooled, ctypes.c_void_p(256 + 16), 1 << 30) == INVALID
        assert scores(pooled, one, exact_scores - 256) == TOO_SMALL
    # a pooling window the matrix-core kernel does not fuse runs on the plain kernel: no scratch asked for
    odd = m.Params.make("bf16", 32, 2, 128, pool_len=3, pool_stride=2)
    assert m.workspace_bytes(m.OP_BLOCK_SCORES_POOLED, odd, batch, total, mx) == 0
    assert m.workspace_bytes(m.OP_BLOCK_SCORES, odd, batch, total, mx) == q_scores
    wide = m.Params.make("bf16", 32, 2, 128, cmp_len=32, cmp_stride=8)                   # 8 keys per block: not fused
    assert m.workspace_bytes(m.OP_BLOCK_SCORES_POOLED, wide, batch, total, mx) == 0


def test_no_kernel_uses_private_segment_memory():
    """The build records the compiler's per-kernel resource usage.  A register array that the compiler moves to
    private-segment (scratch) memory costs a hot kernel tens of percent without any sign in the source, so every
    kernel of the library is required to stay in registers."""
    from paper_2509_24663_amd import build
    res = build.kernel_resources()
    if not res:
        pytest.skip("no resource records: the library was not built in this tree")
    assert set(res) == set(build.sources())
    names = [k for per_file in res.values() for k in per_file]
    for must in ("block_scores_mfma_kernel", "attn_tile_kernel", "dec_attn_kernel", "topk_blocks_kernel",
                 "bwd_dq_mfma_kernel", "bwd_dkv_mfma_kernel"):
        assert any(must in n for n in names), must
    for src, per_file in res.items():
        for name, u in per_file.items():
            assert u["ScratchSize"] == 0 and u["VGPRs Spill"] == 0, (src, name, u)


def test_library_sources_allocate_nothing_and_keep_no_state():
    """The boundary's rules, checked on the sources: no allocation or free of device memory, no memory-pool
    tuning, no environment variable, no function-local static state anywhere in the library."""
    csrc = os.path.join(ROOT, "paper_2509_24663_amd", "csrc")
    banned = re.compile(r"\b(hipMalloc\w*|hipFree\w*|hipHostMalloc|hipMemPool\w*|hipDeviceGetDefaultMemPool|getenv|"
                        r"malloc|calloc|realloc)\s*\(")
    static_state = re.compile(r"^\s+static\s+(?!constexpr|const\b|inline|__device__|_assert)[A-Za-z_:<> ]+\s+\w+(\[[^\]]*\])*\s*(=|;)", re.M)
    for name in sorted(os.listdir(csrc)):
        text = open(os.path.join(csrc, name)).read()
        code = re.sub(r"//[^\n]*|/\*.*?\*/", "", text, flags=re.S)
        assert not banned.search(code), (name, banned.search(code).group(0))
        # the one static array a source may hold is the documented, fixed-size device scratch of the entry point
        # for callers that cannot allocate; it is declared at file scope, not inside a function
        assert not static_state.search(code), (name, static_state.search(code).group(0))
