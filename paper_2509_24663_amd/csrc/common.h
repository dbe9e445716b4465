// Shared device/host helpers of the gfx950 InfLLM-V2 attention library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "infllmv2.h"

namespace ifv2 {

constexpr int kBlock = 64;      // selection block B (Sec. 3.2); the kernels are written for 64
constexpr int kMaxGroup = 16;   // largest GQA group size G handled
constexpr int kWave = 64;

// ---------------------------------------------------------------- element types
struct bf16_t { uint16_t bits; };

__host__ __device__ inline float bf16_to_float(uint16_t b) {
    union { uint32_t u; float f; } x;
    x.u = (uint32_t)b << 16;
    return x.f;
}
__host__ __device__ inline uint16_t float_to_bf16(float f) {   // round to nearest even
    union { uint32_t u; float f; } x;
    x.f = f;
    if ((x.u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x.u >> 16) | 0x40u);   // quiet NaN
    uint32_t r = x.u + 0x7fffu + ((x.u >> 16) & 1u);
    return (uint16_t)(r >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
    __device__ static inline float load(const float *p) { return *p; }
    __device__ static inline void store(float *p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
    __device__ static inline float load(const bf16_t *p) { return bf16_to_float(p->bits); }
    __device__ static inline void store(bf16_t *p, float v) { p->bits = float_to_bf16(v); }
};

// ---------------------------------------------------------------- where a query row lives
// Prefill: rows are packed tokens, sequences delimited by cu_seqlens.  Decode: row b is the
// newest token of sequence b, whose caches start at b * kv_batch_stride.
struct RowMap {
    const int32_t *cu;        // prefill: [batch+1] token offsets;          decode: nullptr
    const int32_t *cu_c;      // prefill: [batch+1] compressed-row offsets; decode: nullptr
    const int32_t *ctx;       // decode: [batch] context lengths;           prefill: nullptr
    int32_t batch;
    int32_t total_rows;       // prefill: total tokens; decode: batch
    int32_t num_kv_heads;
    int64_t kv_tok_stride, kv_head_stride, kv_batch_stride;
    int64_t kc_total_c;       // prefill: rows per head plane of kc
    int64_t kc_head_stride;   // decode: elements between (b,h) planes of the kc cache
};

// Max-pooling of Eq. 6 when it is fused into the score kernels (on == 0: scores per compressed key)
struct PoolArgs {
    int on, len, stride, pad;
};

struct RowLoc {
    int32_t seq, pos, len;    // sequence, position of the query inside it, sequence length
    int64_t kv_base;          // element offset of (token 0, head 0) of that sequence in K / V
};

__device__ inline int find_seq(const int32_t *cu, int batch, int row) {
    int lo = 0, hi = batch - 1;     // largest s with cu[s] <= row
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (cu[mid] <= row) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__device__ inline RowLoc locate(const RowMap &m, int row) {
    RowLoc r;
    if (m.ctx) {
        r.seq = row;
        r.len = m.ctx[row];
        r.pos = r.len - 1;
        r.kv_base = (int64_t)row * m.kv_batch_stride;
    } else {
        r.seq = find_seq(m.cu, m.batch, row);
        int a = m.cu[r.seq];
        r.len = m.cu[r.seq + 1] - a;
        r.pos = row - a;
        r.kv_base = (int64_t)a * m.kv_tok_stride;
    }
    return r;
}

// first compressed key of (sequence, kv head) in the kc array, head_dim d
__device__ inline const float *kc_base(const RowMap &m, const float *kc, int seq, int h, int d) {
    if (m.ctx) return kc + ((int64_t)seq * m.num_kv_heads + h) * m.kc_head_stride;
    return kc + ((int64_t)h * m.kc_total_c + m.cu_c[seq]) * d;
}
// flat index of (kv head h, row) in per-(head,row) outputs: [hkv, T, *] for prefill, [batch, hkv, *] for decode
__device__ inline int64_t head_row(const RowMap &m, int h, int row) {
    return m.ctx ? (int64_t)row * m.num_kv_heads + h : (int64_t)h * m.total_rows + row;
}
// flat index of (query head qh, row) in lse: [hq, T] for prefill, [batch, hq] for decode
__device__ inline int64_t qhead_row(const RowMap &m, int qh, int hq, int row) {
    return m.ctx ? (int64_t)row * hq + qh : (int64_t)qh * m.total_rows + row;
}

__host__ __device__ inline int num_cmp(int n, int lc, int sc) { return n < lc ? 0 : (n - lc) / sc + 1; }
__host__ __device__ inline int visible_cmp(int t, int lc, int sc) { return t < lc - 1 ? 0 : (t - lc + 1) / sc + 1; }

// ---------------------------------------------------------------- wave helpers
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

// ---------------------------------------------------------------- launchers implemented per stage
struct Launch {
    const infllmv2_params *p;
    RowMap map;
    hipStream_t stream;
    int32_t max_len;          // longest sequence (host knowledge, for grid sizing)
    void *ws;                 // caller's scratch (device, 256-byte aligned) and its size
    size_t ws_bytes;
};

int launch_cu_c(const infllmv2_params *p, const int32_t *cu_d, int batch, int32_t *cu_c_d, hipStream_t s);
int launch_compress_k(const Launch &L, const void *k, float *kc, int64_t total_c_rows);
int launch_compress_k_append(const infllmv2_params *p, const void *k, int64_t kv_batch_stride, int64_t kv_head_stride,
                             int64_t kv_tok_stride, float *kc, int64_t kc_head_stride, const int32_t *prev_d,
                             const int32_t *ctx_d, int batch, int max_new, hipStream_t stream);
// cu_h: host cu_seqlens for the tiled kernels' grid (nullptr: single-row / decode form)
// pooled: the output holds one value per selection block (Eq. 6 applied on chip) instead of one per compressed
// key; entry j of a row is written iff its pooling window has a visible key, max(stride j - pad, 0) < v(t)
int launch_block_scores(const Launch &L, const void *q, const float *kc, float *s_out, int64_t row_stride,
                        const int32_t *cu_h, bool pooled);
// pooled: s_in holds block scores as written by launch_block_scores(pooled = true)
int launch_topk(const Launch &L, const float *s_in, int64_t row_stride, int32_t *idx, bool pooled);
// idx == nullptr: dense for every sequence; dense_below: sequences shorter than this are dense anyway
int launch_attn(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx,
                int dense_below, void *out, float *lse, const int32_t *cu_h);

// gradients of stage 4 (idx == nullptr: dense for every sequence); dk, dv float32 [hkv, T, d], zeroed inside
int launch_attn_bwd(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx, int dense_below,
                    const void *out, const float *lse, const void *dout, void *dq, float *dk, float *dv,
                    const int32_t *cu_h);

inline int hip_status(hipError_t e) { return e == hipSuccess ? INFLLMV2_OK : INFLLMV2_ERR_HIP; }

inline size_t align256(size_t x) { return (x + 255) / 256 * 256; }

// ---------------------------------------------------------------- caller-provided scratch
// What a call needs depends on the batch only through a few totals, so the exact need of a call (from its host
// cu_seqlens) and the bound the workspace query returns (from batch, total tokens, longest sequence) share one
// formula each.  All sizes are multiples of 256 bytes; 0 = the path that serves these parameters needs none.
struct BatchTotals {
    int64_t rows;         // tokens
    int64_t blocks;       // sum over sequences of ceil(len / 64)
    int64_t kt_fine;      // sum of ceil(nc(len) / 64): 64-key tiles of K^{C1}
    int64_t kt_coarse;    // the same for the coarse keys of the LSE Approximation
    int64_t sel_words;    // sum of ceil(len / 64) * ceil(len / 32): words of the backward's selection bitmap per KV head
};
BatchTotals exact_totals(const infllmv2_params *p, const int32_t *cu_h, int batch);
BatchTotals bound_totals(const infllmv2_params *p, int batch, int64_t total_tokens, int32_t max_seqlen);
size_t scores_ws_bytes(const infllmv2_params *p, const BatchTotals &t, bool pooled);
size_t attn_fwd_ws_bytes(const infllmv2_params *p, const BatchTotals &t);
// with_bitmap: including the block-major selection bitmap that speeds up dK/dV when block lists are given
size_t attn_bwd_ws_bytes(const infllmv2_params *p, const BatchTotals &t, bool with_bitmap);

}  // namespace ifv2
