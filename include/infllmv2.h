/*
 * infllmv2.h -- C ABI of the MI355X (gfx950) implementation of InfLLM-V2's
 * dense-sparse switchable attention (arXiv 2509.24663).
 *
 * The path has four stages (Sec. 3.2-3.4 of the paper):
 *   1. infllmv2_compress_k      mean-pool keys into compressed keys K^{C1}            (Eq. 3)
 *      infllmv2_compress_k_append   the same for the rows a growing cache has just completed
 *   2. infllmv2_block_scores    softmax(scale * Q K^{C1 T}) summed over the GQA group (Eq. 4, 5, Alg. 1;
 *                               optionally with the LSE Approximation of Sec. 3.4)
 *   3. infllmv2_topk_blocks     max-pool to selection blocks, keep init + local,
 *                               top-k of the rest                                     (Eq. 6, Eq. 2)
 *   4. infllmv2_sparse_attn_fwd causal attention over the selected 64-token blocks of
 *                               the shared K/V (Appendix Alg. 2), dense below the
 *                               length threshold (Sec. 3.2, "switch")
 *      infllmv2_dense_attn_fwd  causal GQA attention                                  (Eq. 1, Appendix Alg. 3)
 *      infllmv2_sparse_decode   stages 2-4 for the one newest token of each sequence
 *                               against K/V and K^{C1} caches
 *
 * General rules
 *   - Every pointer named *_d or documented "device" is GPU memory on the current
 *     HIP device; pointers named *_h are host memory and are only read during the
 *     call.  The library keeps no state and never synchronises: all work is
 *     enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream).  The library allocates nothing and reads no environment variable.  The
 *     caller owns every buffer, including the scratch some calls need, and keeps it
 *     alive until the stream work has finished.  Calls are thread-safe.
 *   - Scratch: calls with a (workspace_d, workspace_bytes) pair take device memory,
 *     256-byte aligned, of at least the size the call needs for its cu_seqlens; its
 *     contents mean nothing before or after the call.  infllmv2_workspace_bytes
 *     returns a sufficient size from the batch's totals alone.  A call that needs no
 *     scratch for its parameters (the query then returns 0) accepts NULL / 0; one
 *     that does returns INFLLMV2_ERR_INVALID_ARGUMENT for a NULL or misaligned
 *     pointer and INFLLMV2_ERR_WORKSPACE_TOO_SMALL for too few bytes, before
 *     anything is launched.  Two calls that run concurrently need separate scratch.
 *   - All indices are 0-based.  Token t of a sequence lies in block t / block_size.
 *     Sequences are packed along the token axis; cu_seqlens has batch+1 int32
 *     entries (cu_seqlens[0] = 0, non-decreasing) and is passed twice: as a host
 *     array (launch geometry, validation) and as a device array (read by kernels).
 *   - Q and O are token-major [total_tokens, num_q_heads, head_dim], contiguous.
 *     Query head g belongs to KV head g / (num_q_heads / num_kv_heads).
 *     K and V are addressed as  base + token * kv_tok_stride + kv_head * kv_head_stride
 *     (strides in elements, head_dim contiguous), so both token-major
 *     [T, hkv, d] and head-major [hkv, T, d] work; head-major keeps a 64-token
 *     block in one contiguous 16 KB run and is the fast layout.
 *   - dtype selects the element type of Q, K, V, O only.  K^{C1}, scores and lse
 *     are always float32; block indices are int32.
 *   - A call with zero total tokens (or batch 0) is a no-op that returns INFLLMV2_OK; data pointers may
 *     then be NULL.
 *   - Return value: INFLLMV2_OK (0) or a negative infllmv2_status.  Arguments are
 *     validated before anything is launched (so validation errors can be tested
 *     without a GPU); a launch failure is reported as INFLLMV2_ERR_HIP.  No
 *     exception crosses this boundary and nothing aborts.
 */
#ifndef INFLLMV2_H
#define INFLLMV2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define INFLLMV2_FP32 0
#define INFLLMV2_BF16 1

typedef enum infllmv2_status {
    INFLLMV2_OK = 0,
    INFLLMV2_ERR_INVALID_ARGUMENT = -1,   /* null pointer, inconsistent sizes, bad cu_seqlens ...      */
    INFLLMV2_ERR_UNSUPPORTED = -2,        /* dtype / head_dim / parameter combination not implemented   */
    INFLLMV2_ERR_WORKSPACE_TOO_SMALL = -3,
    INFLLMV2_ERR_HIP = -4                 /* a HIP call or kernel launch failed                          */
} infllmv2_status;

/* Hyper-parameters in the paper's notation (Sec. 3.2, 3.3; values of Sec. 4.1 in brackets). */
typedef struct infllmv2_params {
    int32_t dtype;            /* INFLLMV2_FP32 or INFLLMV2_BF16: element type of Q, K, V, O                */
    int32_t num_q_heads;      /* h_q  [32]                                                                 */
    int32_t num_kv_heads;     /* h_kv [2]; h_q % h_kv == 0, G = h_q / h_kv <= 16                           */
    int32_t head_dim;         /* d_h  [128]; 64 or 128                                                     */
    int32_t block_size;       /* B    [64]; must be 64                                                     */
    int32_t cmp_len;          /* l_C1 [32]                                                                 */
    int32_t cmp_stride;       /* s_C1 [16]; 1 <= s_C1 <= l_C1                                              */
    int32_t pool_len;         /* l    [5]                                                                  */
    int32_t pool_stride;      /* s    [4]                                                                  */
    int32_t pool_pad;         /* 0: block j pools compressed keys [s*j, s*j+l) as printed in Eq. 6;
                                 p > 0 shifts the window to [s*j-p, s*j-p+l)                               */
    int32_t n_init;           /* |I_init|  [1]                                                             */
    int32_t n_local;          /* |I_local| [32]; >= 1 (the query's own block is always kept)               */
    int32_t topk_total;       /* |I|       [96]; n_init + n_local <= topk_total <= 1024                    */
    int32_t dense_threshold;  /* sequences with fewer tokens than this run dense attention                 */
    float   softmax_scale;    /* multiplies the logits in stage 2 and in attention; 1/sqrt(d_h)            */
    int32_t lse_mode;         /* stage 2 normalisation.  0: exact, both passes of Alg. 1 over K^{C1}.
                               * 1: LSE Approximation (Sec. 3.4, Eq. 7): the log-sum-exp of pass 1 is taken
                               *    over K^{C2} (window 4 l_C1, stride 4 s_C1, formed inside the library from
                               *    K^{C1}; needs l_C1 % s_C1 == 0, else UNSUPPORTED) and used as it is; a row
                               *    that sees no K^{C2} key gets all-zero scores.                              */
} infllmv2_params;

/* Number of compressed keys of a sequence of n tokens: complete windows only,
 * nc(n) = n < l_C1 ? 0 : (n - l_C1) / s_C1 + 1.  Host helper, no GPU needed. */
int32_t infllmv2_num_cmp(const infllmv2_params *p, int32_t n);

/* Human-readable text for a status code (static storage, never NULL). */
const char *infllmv2_status_string(int status);

/* Library version string, e.g. "infllmv2-gfx950 0.2". */
const char *infllmv2_version(void);

/* The calls, as `op` of infllmv2_workspace_bytes. */
typedef enum infllmv2_op {
    INFLLMV2_OP_COMPRESS_K = 0,
    INFLLMV2_OP_BLOCK_SCORES = 1,
    INFLLMV2_OP_TOPK_BLOCKS = 2,
    INFLLMV2_OP_SPARSE_ATTN_FWD = 3,
    INFLLMV2_OP_DENSE_ATTN_FWD = 4,
    INFLLMV2_OP_SPARSE_DECODE = 5,
    INFLLMV2_OP_BLOCK_SCORES_POOLED = 6,
    INFLLMV2_OP_TOPK_POOLED = 7,
    INFLLMV2_OP_SPARSE_ATTN_BWD = 8,        /* including the selection bitmap (see infllmv2_sparse_attn_bwd) */
    INFLLMV2_OP_SPARSE_ATTN_BWD_MIN = 9,    /* without it */
    INFLLMV2_OP_COMPRESS_K_APPEND = 10
} infllmv2_op;

/*
 * Bytes of scratch that call `op` needs at most for any batch of `batch` sequences with total_tokens tokens in
 * all and none longer than max_seqlen (for INFLLMV2_OP_SPARSE_DECODE: `batch` sequences with contexts of at most
 * max_seqlen tokens; total_tokens is ignored).  The inputs of Alg. 1 and Appendix Alg. 2 / 3 and their outputs
 * live in HBM buffers of the caller; so does everything the kernels keep between their launches: a transposed
 * copy of V for the attention calls, a half-precision copy of the compressed keys for the score calls, K^T and
 * per-row terms for the backward call, partial results for decode.  Returns 0 for calls that need none, and 0
 * for parameters that infllmv2_* calls reject.  Host helper, no GPU needed.
 */
size_t infllmv2_workspace_bytes(int op, const infllmv2_params *p, int32_t batch, int64_t total_tokens,
                                int32_t max_seqlen);

/*
 * Stage 1 -- Sec. 3.3, Eq. 3:  K^{C1}_i = Mean(K[i*s_C1 : i*s_C1 + l_C1]) per sequence and KV head.
 *   k              device, dtype elements, addressed with the K/V strides
 *   cu_seqlens_h/d host / device [batch+1]
 *   kc_d           device out, float32 [num_kv_heads, total_c, head_dim] where
 *                  total_c = sum over sequences of nc(len); sequence s starts at row cu_seqlens_c[s]
 *   cu_seqlens_c_d device out, int32 [batch+1], prefix sums of nc(len)
 *   total_c        rows allocated per head in kc_d (>= the sum above, else INVALID_ARGUMENT)
 */
int infllmv2_compress_k(const infllmv2_params *p, const void *k_d, int64_t kv_tok_stride, int64_t kv_head_stride,
                        const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch,
                        float *kc_d, int32_t *cu_seqlens_c_d, int64_t total_c, void *stream);

/*
 * Stage 1 for a growing cache (decode): Sec. 3.3, Eq. 3 applied to the tail of each sequence.  Sequence b had
 * prev_lens[b] tokens in its K cache when its compressed-key cache was last brought up to date and has
 * ctx_lens[b] >= prev_lens[b] now; this writes the compressed keys that became complete in between, rows
 * nc(prev_lens[b]) .. nc(ctx_lens[b]) - 1 of every KV head's plane (one new row every s_C1 tokens), and leaves
 * the other rows alone.  The result equals infllmv2_compress_k on the first ctx_lens[b] tokens.
 *   k_cache_d      device, dtype, token t of (b, h) at  base + b * kv_batch_stride + h * kv_head_stride + t * kv_tok_stride
 *   kc_cache_d     device in/out, float32; plane (b, h) at  base + (b * num_kv_heads + h) * kc_head_stride,
 *                  row i at + i * head_dim  (kc_head_stride >= max_b nc(ctx_lens[b]) * head_dim, else INVALID_ARGUMENT)
 *   prev_lens_h/d, ctx_lens_h/d   host / device int32 [batch]
 */
int infllmv2_compress_k_append(const infllmv2_params *p, const void *k_cache_d, int64_t kv_batch_stride,
                               int64_t kv_head_stride, int64_t kv_tok_stride, float *kc_cache_d, int64_t kc_head_stride,
                               const int32_t *prev_lens_h, const int32_t *prev_lens_d, const int32_t *ctx_lens_h,
                               const int32_t *ctx_lens_d, int32_t batch, void *stream);

/*
 * Stage 2 -- Sec. 3.3 Eq. 4-5, computed as in Alg. 1 (two passes, head-group sum on chip):
 *   for token t (position within its sequence) and KV head h, over the v(t) compressed keys whose
 *   window ends at or before t (v(t) = t < l_C1-1 ? 0 : (t-l_C1+1)/s_C1 + 1):
 *       S^shared[h, t, i] = sum over the G heads g of group h of softmax_i(scale * <Q[t,g], K^{C1}[h,i]>)
 *   q_d            device [total_tokens, num_q_heads, head_dim]
 *   kc_d, cu_seqlens_c_d   as written by infllmv2_compress_k
 *   s_shared_d     device out float32 [num_kv_heads, total_tokens, row_stride]; entries i < v(t) are
 *                  written, the rest of each row is left untouched.  row_stride >= max over sequences
 *                  of nc(len) and a multiple of 4.
 *   workspace_d    device scratch, see the general rules (INFLLMV2_OP_BLOCK_SCORES)
 *   Per-head score matrices never reach HBM; only the group sums are stored.
 */
int infllmv2_block_scores(const infllmv2_params *p, const void *q_d, const float *kc_d, int64_t total_c,
                          const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d,
                          const int32_t *cu_seqlens_c_d, int32_t batch,
                          float *s_shared_d, int64_t row_stride, void *workspace_d, size_t workspace_bytes,
                          void *stream);

/*
 * Stage 3 -- Sec. 3.3 Eq. 6 then Sec. 3.2 Eq. 2, per token t (block b_t = t / B) and KV head:
 *   S^cmp_j = max S^shared[s*j - pad : s*j - pad + l] clipped to the v(t) visible keys (empty -> 0), j <= b_t
 *   forced  = {0..n_init-1} U {b_t-n_local+1..b_t}, clipped to [0, b_t]
 *   top-k   = the min(topk_total - n_init - n_local, #others) other blocks with the largest S^cmp,
 *             equal scores resolved towards the smaller block index
 *   block_idx_d    device out int32 [num_kv_heads, total_tokens, topk_total]: the union, ascending,
 *                  padded with -1.
 */
int infllmv2_topk_blocks(const infllmv2_params *p, const float *s_shared_d, int64_t row_stride,
                         const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch,
                         int32_t *block_idx_d, void *stream);

/*
 * Stages 2 and 3 with the max-pooling of Eq. 6 moved into the score kernel (the fusion Sec. 3.4 names as future
 * work): the group scores never reach memory per compressed key, only per selection block, a buffer
 * pool_stride times smaller than S^shared, and the selection reads that.  The resulting block_idx is identical
 * to infllmv2_block_scores followed by infllmv2_topk_blocks.
 *   s_cmp_d        device float32 [num_kv_heads, total_tokens, row_stride], row_stride >= ceil(max len / 64).
 *                  infllmv2_block_scores_pooled writes S^cmp[h, t, j] = max of S^shared[h, t, i] over
 *                  i in [s*j - pad, s*j - pad + l) clipped to [0, v(t)) for every block j <= b_t whose clipped
 *                  window is not empty, i.e. max(s*j - pad, 0) < v(t), and leaves the other entries untouched;
 *                  infllmv2_topk_pooled reads exactly those entries and takes the others as 0.
 *   Other arguments as for infllmv2_block_scores / infllmv2_topk_blocks (scratch: INFLLMV2_OP_BLOCK_SCORES_POOLED).
 *   Every pooling window is accepted; the paper's (l = 5, s = 4, pad 0 or 1, with s * s_C1 = B) with the paper's head
 *   shape in bfloat16 runs on the matrix cores.
 */
int infllmv2_block_scores_pooled(const infllmv2_params *p, const void *q_d, const float *kc_d, int64_t total_c,
                                 const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d,
                                 const int32_t *cu_seqlens_c_d, int32_t batch,
                                 float *s_cmp_d, int64_t row_stride, void *workspace_d, size_t workspace_bytes,
                                 void *stream);
int infllmv2_topk_pooled(const infllmv2_params *p, const float *s_cmp_d, int64_t row_stride,
                         const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch,
                         int32_t *block_idx_d, void *stream);

/*
 * Stage 4 -- Appendix Alg. 2: token t attends, with one softmax per query head, to the keys u <= t
 * whose block u / B is listed in block_idx[h, t, :]; O = softmax(scale * q K^T) V.
 * Sequences shorter than dense_threshold ignore block_idx and attend to every u <= t (Sec. 3.2).
 *   block_idx_d    device int32 [num_kv_heads, total_tokens, topk_total] (entries must be valid block
 *                  numbers <= b_t or -1; as produced by infllmv2_topk_blocks)
 *   out_d          device out, dtype [total_tokens, num_q_heads, head_dim]
 *   lse_d          device out float32 [num_q_heads, total_tokens]: ln sum_u exp(scale * <q, k_u>); may be NULL
 *   workspace_d    device scratch, see the general rules (INFLLMV2_OP_SPARSE_ATTN_FWD)
 */
int infllmv2_sparse_attn_fwd(const infllmv2_params *p, const void *q_d, const void *k_d, const void *v_d,
                             int64_t kv_tok_stride, int64_t kv_head_stride, const int32_t *block_idx_d,
                             const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch,
                             void *out_d, float *lse_d, void *workspace_d, size_t workspace_bytes, void *stream);

/*
 * Gradients of stage 4 with respect to Q, K and V for a given selection.  The paper trains through this
 * attention (Sec. 3.2; Alg. 2 returns the log-sum-exp for that purpose) but prints no backward algorithm: this is
 * the chain rule on O = softmax(scale * q K^T) V over the keys stage 4 attends to.  The selection only picks
 * blocks (Sec. 3.3), so nothing flows back into stages 1-3.
 *   block_idx_d    as for infllmv2_sparse_attn_fwd, or NULL: every sequence attends densely (Eq. 1)
 *   out_d, lse_d   device, what the forward call produced from the same inputs
 *   dout_d         device, dtype [total_tokens, num_q_heads, head_dim]: gradient of the loss w.r.t. out
 *   dq_d           device out, dtype [total_tokens, num_q_heads, head_dim]
 *   dk_d, dv_d     device out, float32 [num_kv_heads, total_tokens, head_dim], 16-byte aligned, ordinary
 *                  (coarse-grained, hipMalloc-style) device memory; overwritten.  Each row sums the
 *                  contributions of the num_q_heads / num_kv_heads heads of its group and of every query row
 *                  that attends to it; they are added up with the L2's float atomics, so the last bits may
 *                  differ between runs.
 *   workspace_d    device scratch, see the general rules.  INFLLMV2_OP_SPARSE_ATTN_BWD_MIN bytes are required.
 *                  For bf16 data with 16 query heads per KV head and head_dim 128 (the matrix-core path) a
 *                  workspace of INFLLMV2_OP_SPARSE_ATTN_BWD bytes also has room for a selection bitmap of
 *                  num_kv_heads * sum over sequences of ceil(len / 64) * ceil(len / 32) words (32 MB per KV head for
 *                  one 128K-token sequence), which the call then builds and which makes dK / dV faster; with less it
 *                  searches the block lists instead: same results.
 */
int infllmv2_sparse_attn_bwd(const infllmv2_params *p, const void *q_d, const void *k_d, const void *v_d,
                             int64_t kv_tok_stride, int64_t kv_head_stride, const int32_t *block_idx_d,
                             const void *out_d, const float *lse_d, const void *dout_d,
                             const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch,
                             void *dq_d, float *dk_d, float *dv_d, void *workspace_d, size_t workspace_bytes,
                             void *stream);

/* Dense causal GQA attention -- Eq. 1 (tile schedule of Appendix Alg. 3).  Arguments as for
 * infllmv2_sparse_attn_fwd (scratch: INFLLMV2_OP_DENSE_ATTN_FWD). */
int infllmv2_dense_attn_fwd(const infllmv2_params *p, const void *q_d, const void *k_d, const void *v_d,
                            int64_t kv_tok_stride, int64_t kv_head_stride,
                            const int32_t *cu_seqlens_h, const int32_t *cu_seqlens_d, int32_t batch,
                            void *out_d, float *lse_d, void *workspace_d, size_t workspace_bytes, void *stream);

/*
 * Decode step -- stages 2-4 for the single query row t = ctx_len-1 of every sequence (the paper
 * states decode support, Sec. 2.2 / 4.3, without a separate algorithm; it is that row of the prefill).
 *   q_d            device [batch, num_q_heads, head_dim]
 *   k_cache_d, v_cache_d   device, element (b, h, t, c) at
 *                  base + b*kv_batch_stride + h*kv_head_stride + t*kv_tok_stride + c; the newest
 *                  token's K/V are already stored at t = ctx_len-1
 *   kc_cache_d     device float32, row i of (b, h) at base + (b*num_kv_heads + h)*kc_head_stride + i*head_dim;
 *                  holds at least nc(ctx_len) rows
 *   ctx_lens_h/d   host / device int32 [batch], each >= 1
 *   block_idx_out_d device out int32 [batch, num_kv_heads, topk_total] or NULL
 *   out_d          device out dtype [batch, num_q_heads, head_dim];  lse_d float32 [batch, num_q_heads] or NULL
 *   workspace_d    device scratch of at least infllmv2_decode_workspace_bytes(...) bytes, 256-byte aligned
 * Contexts longer than 262144 tokens are supported only for bf16 data with 16 query heads per KV head and
 * head_dim 128 (with the LSE Approximation up to about 419000 tokens; longer ones return INFLLMV2_ERR_UNSUPPORTED).
 * Sequences shorter than dense_threshold attend densely.
 */
int infllmv2_sparse_decode(const infllmv2_params *p, const void *q_d, const void *k_cache_d, const void *v_cache_d,
                           int64_t kv_batch_stride, int64_t kv_head_stride, int64_t kv_tok_stride,
                           const float *kc_cache_d, int64_t kc_head_stride,
                           const int32_t *ctx_lens_h, const int32_t *ctx_lens_d, int32_t batch,
                           int32_t *block_idx_out_d, void *out_d, float *lse_d,
                           void *workspace_d, size_t workspace_bytes, void *stream);

/* Bytes of scratch infllmv2_sparse_decode needs for `batch` sequences of at most max_ctx_len tokens
 * (= infllmv2_workspace_bytes(INFLLMV2_OP_SPARSE_DECODE, p, batch, 0, max_ctx_len)). */
size_t infllmv2_decode_workspace_bytes(const infllmv2_params *p, int32_t batch, int32_t max_ctx_len);

/*
 * infllmv2_sparse_decode for callers that cannot allocate or pass device scratch: code under HIP graph capture that
 * may not call hipMalloc, tight serving loops, harnesses that forbid allocation.  Same arguments, results and
 * errors as infllmv2_sparse_decode without (workspace_d, workspace_bytes): the scratch is a fixed array of
 * infllmv2_sparse_decode_static_capacity() bytes (16 MiB: batch 16 with contexts up to 65536 tokens fits) inside the
 * library's device image, which every GPU the library runs on holds until the process ends.  A step that needs
 * more (infllmv2_decode_workspace_bytes) returns INFLLMV2_ERR_WORKSPACE_TOO_SMALL before anything is launched.  The
 * call allocates and frees nothing.  All calls on one GPU share that GPU's array: calls that overlap in time on one
 * GPU (different streams or threads) race and give undefined results; calls on one stream, or ordered by events,
 * are fine.  The first call on a GPU looks the array's address up once (a host-side query).
 */
int infllmv2_sparse_decode_static(const infllmv2_params *p, const void *q_d, const void *k_cache_d,
                                  const void *v_cache_d, int64_t kv_batch_stride, int64_t kv_head_stride,
                                  int64_t kv_tok_stride, const float *kc_cache_d, int64_t kc_head_stride,
                                  const int32_t *ctx_lens_h, const int32_t *ctx_lens_d, int32_t batch,
                                  int32_t *block_idx_out_d, void *out_d, float *lse_d, void *stream);
size_t infllmv2_sparse_decode_static_capacity(void);

#ifdef __cplusplus
}
#endif
#endif /* INFLLMV2_H */
