// C ABI entry points: argument validation (host only, before any launch) and dispatch to the kernels.
#include <math.h>

#include "common.h"

using namespace ifv2;

namespace ifv2 {
int launch_attn_generic(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx,
                        int dense_below, void *out, float *lse);
int launch_attn_mfma(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx,
                     int dense_below, void *out, float *lse, const int32_t *cu_h);
bool attn_mfma_supported(const infllmv2_params *p);
bool decode_mfma_supported(const infllmv2_params *p);
size_t decode_mfma_workspace(const infllmv2_params *p, int batch, int max_ctx);
int launch_decode_mfma(const infllmv2_params *p, const void *q, const void *k, const void *v, int64_t kv_batch_stride,
                       int64_t kv_head_stride, int64_t kv_tok_stride, const float *kc, int64_t kc_head_stride,
                       const int32_t *ctx_h, const int32_t *ctx_d, int batch, int32_t *idx_out, void *out, float *lse,
                       void *ws, hipStream_t stream);
}  // namespace ifv2

static int check_params(const infllmv2_params *p) {
    if (p == nullptr) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (p->dtype != INFLLMV2_FP32 && p->dtype != INFLLMV2_BF16) return INFLLMV2_ERR_UNSUPPORTED;
    if (p->num_q_heads <= 0 || p->num_kv_heads <= 0 || p->num_q_heads % p->num_kv_heads != 0)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (p->num_q_heads / p->num_kv_heads > kMaxGroup) return INFLLMV2_ERR_UNSUPPORTED;
    if (p->head_dim != 64 && p->head_dim != 128) return INFLLMV2_ERR_UNSUPPORTED;
    if (p->block_size != kBlock) return INFLLMV2_ERR_UNSUPPORTED;
    if (p->cmp_stride < 1 || p->cmp_len < p->cmp_stride) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (p->pool_len < 1 || p->pool_stride < 1 || p->pool_pad < 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (p->n_init < 0 || p->n_local < 1) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (p->topk_total < p->n_init + p->n_local) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (p->topk_total > 1024) return INFLLMV2_ERR_UNSUPPORTED;
    if (p->dense_threshold < 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (!(p->softmax_scale > 0.f) || !isfinite(p->softmax_scale)) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (p->lse_mode != 0 && p->lse_mode != 1) return INFLLMV2_ERR_INVALID_ARGUMENT;
    // the coarse keys of the LSE Approximation are formed from whole K^{C1} windows
    if (p->lse_mode == 1 && p->cmp_len % p->cmp_stride != 0) return INFLLMV2_ERR_UNSUPPORTED;
    return INFLLMV2_OK;
}

// cu_seqlens: [batch+1], starts at 0, non-decreasing.  Returns total tokens / longest sequence.
static int check_cu(const int32_t *cu_h, const int32_t *cu_d, int32_t batch, int64_t *total, int32_t *max_len) {
    if (cu_h == nullptr || cu_d == nullptr || batch < 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (cu_h[0] != 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    int32_t mx = 0;
    for (int s = 0; s < batch; ++s) {
        if (cu_h[s + 1] < cu_h[s]) return INFLLMV2_ERR_INVALID_ARGUMENT;
        int32_t len = cu_h[s + 1] - cu_h[s];
        if (len > mx) mx = len;
    }
    *total = cu_h[batch];
    *max_len = mx;
    return INFLLMV2_OK;
}

// workspace arguments: 256-byte aligned when present; need == 0 accepts anything (also NULL)
static int check_ws(const void *ws, size_t ws_bytes, size_t need) {
    if (need == 0) return INFLLMV2_OK;
    if (ws == nullptr || ((uintptr_t)ws & 255) != 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    return ws_bytes < need ? INFLLMV2_ERR_WORKSPACE_TOO_SMALL : INFLLMV2_OK;
}

static RowMap prefill_map(const infllmv2_params *p, const int32_t *cu_d, const int32_t *cu_c_d, int batch,
                          int64_t total, int64_t tok_stride, int64_t head_stride, int64_t kc_total_c) {
    RowMap m;
    m.cu = cu_d;
    m.cu_c = cu_c_d;
    m.ctx = nullptr;
    m.batch = batch;
    m.total_rows = (int32_t)total;
    m.num_kv_heads = p->num_kv_heads;
    m.kv_tok_stride = tok_stride;
    m.kv_head_stride = head_stride;
    m.kv_batch_stride = 0;
    m.kc_total_c = kc_total_c;
    m.kc_head_stride = 0;
    return m;
}

extern "C" {

int32_t infllmv2_num_cmp(const infllmv2_params *p, int32_t n) {
    if (p == nullptr || p->cmp_stride < 1 || n < 0) return 0;
    return num_cmp(n, p->cmp_len, p->cmp_stride);
}

const char *infllmv2_status_string(int status) {
    switch (status) {
        case INFLLMV2_OK: return "ok";
        case INFLLMV2_ERR_INVALID_ARGUMENT: return "invalid argument";
        case INFLLMV2_ERR_UNSUPPORTED: return "unsupported dtype, head shape or parameter";
        case INFLLMV2_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case INFLLMV2_ERR_HIP: return "HIP error (launch or runtime call failed)";
        default: return "unknown status";
    }
}

const char *infllmv2_version(void) { return "infllmv2-gfx950 0.2"; }

int infllmv2_compress_k(const infllmv2_params *p, const void *k_d, int64_t kv_tok_stride, int64_t kv_head_stride,
                        const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch,
                        float *kc_d, int32_t *cu_seqlens_c_d, int64_t total_c, void *stream) {
    int st = check_params(p);
    if (st) return st;
    int64_t total;
    int32_t max_len;
    st = check_cu(cu_seqlens_h, cu_seqlens_d, batch, &total, &max_len);
    if (st) return st;
    if (cu_seqlens_c_d == nullptr) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (total == 0) return launch_cu_c(p, cu_seqlens_d, batch, cu_seqlens_c_d, (hipStream_t)stream);
    if (k_d == nullptr || kc_d == nullptr) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (kv_tok_stride < p->head_dim || kv_head_stride < p->head_dim) return INFLLMV2_ERR_INVALID_ARGUMENT;
    int64_t need = 0;
    for (int s = 0; s < batch; ++s) need += num_cmp(cu_seqlens_h[s + 1] - cu_seqlens_h[s], p->cmp_len, p->cmp_stride);
    if (total_c < need || total_c >= (1ll << 31)) return INFLLMV2_ERR_INVALID_ARGUMENT;
    hipStream_t s = (hipStream_t)stream;
    st = launch_cu_c(p, cu_seqlens_d, batch, cu_seqlens_c_d, s);
    if (st) return st;
    Launch L{p, prefill_map(p, cu_seqlens_d, cu_seqlens_c_d, batch, total, kv_tok_stride, kv_head_stride, total_c), s,
             max_len, nullptr, 0};
    return launch_compress_k(L, k_d, kc_d, need);
}

int infllmv2_compress_k_append(const infllmv2_params *p, const void *k_cache_d, int64_t kv_batch_stride,
                               int64_t kv_head_stride, int64_t kv_tok_stride, float *kc_cache_d, int64_t kc_head_stride,
                               const int32_t *prev_lens_h, const int32_t *prev_lens_d, const int32_t *ctx_lens_h,
                               const int32_t *ctx_lens_d, int32_t batch, void *stream) {
    int st = check_params(p);
    if (st) return st;
    if (batch < 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (batch == 0) return INFLLMV2_OK;
    if (prev_lens_h == nullptr || prev_lens_d == nullptr || ctx_lens_h == nullptr || ctx_lens_d == nullptr)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    int max_new = 0, max_nc = 0;
    for (int b = 0; b < batch; ++b) {
        if (prev_lens_h[b] < 0 || ctx_lens_h[b] < prev_lens_h[b]) return INFLLMV2_ERR_INVALID_ARGUMENT;
        const int n1 = num_cmp(ctx_lens_h[b], p->cmp_len, p->cmp_stride);
        const int grown = n1 - num_cmp(prev_lens_h[b], p->cmp_len, p->cmp_stride);
        if (grown > max_new) max_new = grown;
        if (n1 > max_nc) max_nc = n1;
    }
    if (max_new == 0) return INFLLMV2_OK;
    if (k_cache_d == nullptr || kc_cache_d == nullptr) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (kv_tok_stride < p->head_dim || kc_head_stride < (int64_t)max_nc * p->head_dim) return INFLLMV2_ERR_INVALID_ARGUMENT;
    return launch_compress_k_append(p, k_cache_d, kv_batch_stride, kv_head_stride, kv_tok_stride, kc_cache_d,
                                    kc_head_stride, prev_lens_d, ctx_lens_d, batch, max_new, (hipStream_t)stream);
}

int infllmv2_block_scores(const infllmv2_params *p, const void *q_d, const float *kc_d, int64_t total_c,
                          const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d,
                          const int32_t *cu_seqlens_c_d, int32_t batch,
                          float *s_shared_d, int64_t row_stride, void *workspace_d, size_t workspace_bytes,
                          void *stream) {
    int st = check_params(p);
    if (st) return st;
    int64_t total;
    int32_t max_len;
    st = check_cu(cu_seqlens_h, cu_seqlens_d, batch, &total, &max_len);
    if (st) return st;
    if (total == 0) return INFLLMV2_OK;
    if (q_d == nullptr || kc_d == nullptr || cu_seqlens_c_d == nullptr || s_shared_d == nullptr)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (row_stride < num_cmp(max_len, p->cmp_len, p->cmp_stride) || row_stride % 4 != 0 || row_stride < 4)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    st = check_ws(workspace_d, workspace_bytes, scores_ws_bytes(p, exact_totals(p, cu_seqlens_h, batch), false));
    if (st) return st;
    Launch L{p, prefill_map(p, cu_seqlens_d, cu_seqlens_c_d, batch, total, 0, 0, total_c), (hipStream_t)stream,
             max_len, workspace_d, workspace_bytes};
    return launch_block_scores(L, q_d, kc_d, s_shared_d, row_stride, cu_seqlens_h, false);
}

int infllmv2_topk_blocks(const infllmv2_params *p, const float *s_shared_d, int64_t row_stride,
                         const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch,
                         int32_t *block_idx_d, void *stream) {
    int st = check_params(p);
    if (st) return st;
    int64_t total;
    int32_t max_len;
    st = check_cu(cu_seqlens_h, cu_seqlens_d, batch, &total, &max_len);
    if (st) return st;
    if (total == 0) return INFLLMV2_OK;
    if (s_shared_d == nullptr || block_idx_d == nullptr) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (row_stride < num_cmp(max_len, p->cmp_len, p->cmp_stride) || row_stride < 4) return INFLLMV2_ERR_INVALID_ARGUMENT;
    Launch L{p, prefill_map(p, cu_seqlens_d, nullptr, batch, total, 0, 0, 0), (hipStream_t)stream, max_len, nullptr, 0};
    return launch_topk(L, s_shared_d, row_stride, block_idx_d, false);
}

// number of selection blocks of an n-token sequence
static inline int num_blocks(int n) { return (n + kBlock - 1) / kBlock; }

int infllmv2_block_scores_pooled(const infllmv2_params *p, const void *q_d, const float *kc_d, int64_t total_c,
                                 const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d,
                                 const int32_t *cu_seqlens_c_d, int32_t batch,
                                 float *s_cmp_d, int64_t row_stride, void *workspace_d, size_t workspace_bytes,
                                 void *stream) {
    int st = check_params(p);
    if (st) return st;
    int64_t total;
    int32_t max_len;
    st = check_cu(cu_seqlens_h, cu_seqlens_d, batch, &total, &max_len);
    if (st) return st;
    if (total == 0) return INFLLMV2_OK;
    if (q_d == nullptr || kc_d == nullptr || cu_seqlens_c_d == nullptr || s_cmp_d == nullptr)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (row_stride < num_blocks(max_len)) return INFLLMV2_ERR_INVALID_ARGUMENT;
    st = check_ws(workspace_d, workspace_bytes, scores_ws_bytes(p, exact_totals(p, cu_seqlens_h, batch), true));
    if (st) return st;
    Launch L{p, prefill_map(p, cu_seqlens_d, cu_seqlens_c_d, batch, total, 0, 0, total_c), (hipStream_t)stream,
             max_len, workspace_d, workspace_bytes};
    return launch_block_scores(L, q_d, kc_d, s_cmp_d, row_stride, cu_seqlens_h, true);
}

int infllmv2_topk_pooled(const infllmv2_params *p, const float *s_cmp_d, int64_t row_stride,
                         const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch,
                         int32_t *block_idx_d, void *stream) {
    int st = check_params(p);
    if (st) return st;
    int64_t total;
    int32_t max_len;
    st = check_cu(cu_seqlens_h, cu_seqlens_d, batch, &total, &max_len);
    if (st) return st;
    if (total == 0) return INFLLMV2_OK;
    if (s_cmp_d == nullptr || block_idx_d == nullptr) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (row_stride < num_blocks(max_len)) return INFLLMV2_ERR_INVALID_ARGUMENT;
    Launch L{p, prefill_map(p, cu_seqlens_d, nullptr, batch, total, 0, 0, 0), (hipStream_t)stream, max_len, nullptr, 0};
    return launch_topk(L, s_cmp_d, row_stride, block_idx_d, true);
}

static int attn_common(const infllmv2_params *p, const void *q_d, const void *k_d, const void *v_d,
                       int64_t kv_tok_stride, int64_t kv_head_stride, const int32_t *block_idx_d, bool sparse,
                       const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch, void *out_d,
                       float *lse_d, void *workspace_d, size_t workspace_bytes, void *stream) {
    int st = check_params(p);
    if (st) return st;
    int64_t total;
    int32_t max_len;
    st = check_cu(cu_seqlens_h, cu_seqlens_d, batch, &total, &max_len);
    if (st) return st;
    if (total == 0) return INFLLMV2_OK;
    if (q_d == nullptr || k_d == nullptr || v_d == nullptr || out_d == nullptr) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (sparse && block_idx_d == nullptr) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (kv_tok_stride < p->head_dim || kv_head_stride < p->head_dim) return INFLLMV2_ERR_INVALID_ARGUMENT;
    st = check_ws(workspace_d, workspace_bytes, attn_fwd_ws_bytes(p, exact_totals(p, cu_seqlens_h, batch)));
    if (st) return st;
    Launch L{p, prefill_map(p, cu_seqlens_d, nullptr, batch, total, kv_tok_stride, kv_head_stride, 0),
             (hipStream_t)stream, max_len, workspace_d, workspace_bytes};
    return launch_attn(L, q_d, k_d, v_d, sparse ? block_idx_d : nullptr, sparse ? p->dense_threshold : 0, out_d,
                       lse_d, cu_seqlens_h);
}

int infllmv2_sparse_attn_fwd(const infllmv2_params *p, const void *q_d, const void *k_d, const void *v_d,
                             int64_t kv_tok_stride, int64_t kv_head_stride, const int32_t *block_idx_d,
                             const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch,
                             void *out_d, float *lse_d, void *workspace_d, size_t workspace_bytes, void *stream) {
    return attn_common(p, q_d, k_d, v_d, kv_tok_stride, kv_head_stride, block_idx_d, true, cu_seqlens_h,
                       cu_seqlens_d, batch, out_d, lse_d, workspace_d, workspace_bytes, stream);
}

int infllmv2_dense_attn_fwd(const infllmv2_params *p, const void *q_d, const void *k_d, const void *v_d,
                            int64_t kv_tok_stride, int64_t kv_head_stride,
                            const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch,
                            void *out_d, float *lse_d, void *workspace_d, size_t workspace_bytes, void *stream) {
    return attn_common(p, q_d, k_d, v_d, kv_tok_stride, kv_head_stride, nullptr, false, cu_seqlens_h,
                       cu_seqlens_d, batch, out_d, lse_d, workspace_d, workspace_bytes, stream);
}

int infllmv2_sparse_attn_bwd(const infllmv2_params *p, const void *q_d, const void *k_d, const void *v_d,
                             int64_t kv_tok_stride, int64_t kv_head_stride, const int32_t *block_idx_d,
                             const void *out_d, const float *lse_d, const void *dout_d,
                             const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch,
                             void *dq_d, float *dk_d, float *dv_d, void *workspace_d, size_t workspace_bytes,
                             void *stream) {
    int st = check_params(p);
    if (st) return st;
    int64_t total;
    int32_t max_len;
    st = check_cu(cu_seqlens_h, cu_seqlens_d, batch, &total, &max_len);
    if (st) return st;
    if (total == 0) return INFLLMV2_OK;
    if (q_d == nullptr || k_d == nullptr || v_d == nullptr || out_d == nullptr || lse_d == nullptr || dout_d == nullptr ||
        dq_d == nullptr || dk_d == nullptr || dv_d == nullptr)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (kv_tok_stride < p->head_dim || kv_head_stride < p->head_dim) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if ((((uintptr_t)dk_d | (uintptr_t)dv_d) & 15) != 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    st = check_ws(workspace_d, workspace_bytes, attn_bwd_ws_bytes(p, exact_totals(p, cu_seqlens_h, batch), false));
    if (st) return st;
    Launch L{p, prefill_map(p, cu_seqlens_d, nullptr, batch, total, kv_tok_stride, kv_head_stride, 0),
             (hipStream_t)stream, max_len, workspace_d, workspace_bytes};
    return launch_attn_bwd(L, q_d, k_d, v_d, block_idx_d, block_idx_d ? p->dense_threshold : 0, out_d, lse_d, dout_d,
                           dq_d, dk_d, dv_d, cu_seqlens_h);
}

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

size_t infllmv2_workspace_bytes(int op, const infllmv2_params *p, int32_t batch, int64_t total_tokens,
                                int32_t max_seqlen) {
    if (check_params(p) != INFLLMV2_OK || batch < 0 || total_tokens < 0 || max_seqlen < 0) return 0;
    if (op == INFLLMV2_OP_SPARSE_DECODE) return infllmv2_decode_workspace_bytes(p, batch, max_seqlen);
    if (total_tokens >= (1ll << 31)) return 0;
    const BatchTotals t = bound_totals(p, batch, total_tokens, max_seqlen);
    switch (op) {
        case INFLLMV2_OP_BLOCK_SCORES: return scores_ws_bytes(p, t, false);
        case INFLLMV2_OP_BLOCK_SCORES_POOLED: return scores_ws_bytes(p, t, true);
        case INFLLMV2_OP_SPARSE_ATTN_FWD:
        case INFLLMV2_OP_DENSE_ATTN_FWD: return attn_fwd_ws_bytes(p, t);
        case INFLLMV2_OP_SPARSE_ATTN_BWD: return attn_bwd_ws_bytes(p, t, true);
        case INFLLMV2_OP_SPARSE_ATTN_BWD_MIN: return attn_bwd_ws_bytes(p, t, false);
        default: return 0;      // compress_k, compress_k_append, top-k: no scratch
    }
}

size_t infllmv2_decode_workspace_bytes(const infllmv2_params *p, int32_t batch, int32_t max_ctx_len) {
    if (check_params(p) != INFLLMV2_OK || batch < 0 || max_ctx_len < 0) return 0;
    const size_t rs = align_up((size_t)num_cmp(max_ctx_len, p->cmp_len, p->cmp_stride) + 4, 4);
    const size_t rows = (size_t)batch * p->num_kv_heads;
    const size_t generic = align_up(rows * rs * sizeof(float), 256) + align_up(rows * p->topk_total * sizeof(int32_t), 256) + 256;
    const size_t fast = decode_mfma_supported(p) ? decode_mfma_workspace(p, batch, max_ctx_len) : 0;
    return generic > fast ? generic : fast;
}

int infllmv2_sparse_decode(const infllmv2_params *p, const void *q_d, const void *k_cache_d, const void *v_cache_d,
                           int64_t kv_batch_stride, int64_t kv_head_stride, int64_t kv_tok_stride,
                           const float *kc_cache_d, int64_t kc_head_stride,
                           const int32_t *ctx_lens_h, const int32_t *ctx_lens_d, int32_t batch,
                           int32_t *block_idx_out_d, void *out_d, float *lse_d,
                           void *workspace_d, size_t workspace_bytes, void *stream) {
    int st = check_params(p);
    if (st) return st;
    if (q_d == nullptr || k_cache_d == nullptr || v_cache_d == nullptr || kc_cache_d == nullptr ||
        ctx_lens_h == nullptr || ctx_lens_d == nullptr || out_d == nullptr || batch < 0)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (kv_tok_stride < p->head_dim || kv_head_stride < p->head_dim || kv_batch_stride < p->head_dim)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    int32_t max_ctx = 0;
    for (int b = 0; b < batch; ++b) {
        if (ctx_lens_h[b] < 1) return INFLLMV2_ERR_INVALID_ARGUMENT;
        if (ctx_lens_h[b] > max_ctx) max_ctx = ctx_lens_h[b];
    }
    if (kc_head_stride < (int64_t)num_cmp(max_ctx, p->cmp_len, p->cmp_stride) * p->head_dim)
        return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (batch == 0) return INFLLMV2_OK;
    const size_t need = infllmv2_decode_workspace_bytes(p, batch, max_ctx);
    if (workspace_d == nullptr || ((uintptr_t)workspace_d & 255) != 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < need) return INFLLMV2_ERR_WORKSPACE_TOO_SMALL;

    const bool aligned = (((uintptr_t)q_d | (uintptr_t)k_cache_d | (uintptr_t)v_cache_d | (uintptr_t)kc_cache_d |
                           (uintptr_t)out_d) & 15) == 0 &&
                         kv_tok_stride % 8 == 0 && kv_head_stride % 8 == 0 && kv_batch_stride % 8 == 0 &&
                         kc_head_stride % 4 == 0;
    if (decode_mfma_supported(p) && aligned) {
        const int rc = launch_decode_mfma(p, q_d, k_cache_d, v_cache_d, kv_batch_stride, kv_head_stride, kv_tok_stride,
                                          kc_cache_d, kc_head_stride, ctx_lens_h, ctx_lens_d, batch, block_idx_out_d,
                                          out_d, lse_d, workspace_d, (hipStream_t)stream);
        if (rc != INFLLMV2_ERR_UNSUPPORTED) return rc;
    }

    const size_t rs = align_up((size_t)num_cmp(max_ctx, p->cmp_len, p->cmp_stride) + 4, 4);
    const size_t rows = (size_t)batch * p->num_kv_heads;
    float *scores = (float *)workspace_d;
    int32_t *idx_ws = (int32_t *)((char *)workspace_d + align_up(rows * rs * sizeof(float), 256));
    int32_t *idx = block_idx_out_d ? block_idx_out_d : idx_ws;

    RowMap m;
    m.cu = nullptr;
    m.cu_c = nullptr;
    m.ctx = ctx_lens_d;
    m.batch = batch;
    m.total_rows = batch;
    m.num_kv_heads = p->num_kv_heads;
    m.kv_tok_stride = kv_tok_stride;
    m.kv_head_stride = kv_head_stride;
    m.kv_batch_stride = kv_batch_stride;
    m.kc_total_c = 0;
    m.kc_head_stride = kc_head_stride;
    Launch L{p, m, (hipStream_t)stream, max_ctx, nullptr, 0};
    st = launch_block_scores(L, q_d, kc_cache_d, scores, (int64_t)rs, nullptr, false);
    if (st) return st;
    st = launch_topk(L, scores, (int64_t)rs, idx, false);
    if (st) return st;
    return launch_attn_generic(L, q_d, k_cache_d, v_cache_d, idx, p->dense_threshold, out_d, lse_d);
}

}  // extern "C"

namespace ifv2 {
BatchTotals exact_totals(const infllmv2_params *p, const int32_t *cu_h, int batch) {
    BatchTotals t{0, 0, 0, 0, 0};
    for (int s = 0; s < batch; ++s) {
        const int64_t len = cu_h[s + 1] - cu_h[s];
        t.rows += len;
        t.blocks += (len + kBlock - 1) / kBlock;
        t.kt_fine += (num_cmp((int)len, p->cmp_len, p->cmp_stride) + kBlock - 1) / kBlock;
        t.kt_coarse += (num_cmp((int)len, 4 * p->cmp_len, 4 * p->cmp_stride) + kBlock - 1) / kBlock;
        t.sel_words += ((len + kBlock - 1) / kBlock) * ((len + 31) / 32);
    }
    return t;
}

// every total of exact_totals is at most this for any batch of `batch` sequences, total_tokens tokens, none
// longer than max_seqlen (nc(n) <= n / s_C1 because l_C1 >= s_C1)
BatchTotals bound_totals(const infllmv2_params *p, int batch, int64_t total_tokens, int32_t max_seqlen) {
    BatchTotals t;
    t.rows = total_tokens;
    t.blocks = total_tokens / kBlock + batch;
    t.kt_fine = total_tokens / ((int64_t)p->cmp_stride * kBlock) + batch;
    t.kt_coarse = total_tokens / ((int64_t)4 * p->cmp_stride * kBlock) + batch;
    t.sel_words = t.blocks * ((int64_t)max_seqlen / 32 + 1);
    return t;
}

int launch_attn(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx,
                int dense_below, void *out, float *lse, const int32_t *cu_h) {
    const bool aligned = (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15) == 0 &&
                         L.map.kv_tok_stride % 8 == 0 && L.map.kv_head_stride % 8 == 0;
    if (attn_mfma_supported(L.p) && aligned) {
        const int rc = launch_attn_mfma(L, q, k, v, idx, dense_below, out, lse, cu_h);
        if (rc != INFLLMV2_ERR_UNSUPPORTED) return rc;      // strides or sizes outside the tile kernel's limits
    }
    return launch_attn_generic(L, q, k, v, idx, dense_below, out, lse);
}
}  // namespace ifv2
