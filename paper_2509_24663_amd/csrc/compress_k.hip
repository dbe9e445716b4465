// Stage 1: mean-pooled compressed keys, K^{C1}_i = Mean(K[i*s : i*s + l])  (Sec. 3.3, Eq. 3).
// HBM-bound: every K element is needed by l/s (= 2) windows; the second use hits L2.
#include "common.h"

namespace ifv2 {

// prefix sums of the per-sequence compressed-key counts (batch is small: one thread)
__global__ void cu_c_kernel(const int32_t *__restrict__ cu, int batch, int lc, int sc, int32_t *__restrict__ cu_c) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        int acc = 0;
        cu_c[0] = 0;
        for (int s = 0; s < batch; ++s) {
            acc += num_cmp(cu[s + 1] - cu[s], lc, sc);
            cu_c[s + 1] = acc;
        }
    }
}

int launch_cu_c(const infllmv2_params *p, const int32_t *cu_d, int batch, int32_t *cu_c_d, hipStream_t s) {
    hipLaunchKernelGGL(cu_c_kernel, dim3(1), dim3(64), 0, s, cu_d, batch, p->cmp_len, p->cmp_stride, cu_c_d);
    return hip_status(hipGetLastError());
}

// One thread owns 8 consecutive channels of one compressed row and walks the l window rows.
// A wave therefore reads whole 256-byte (bf16, d=128) K rows, fully coalesced.
template <typename T, int D>
__global__ void __launch_bounds__(256)
compress_k_kernel(const T *__restrict__ k, RowMap map, int lc, int sc, int total_c, float *__restrict__ kc) {
    constexpr int VEC = 8, VPR = D / VEC, ROWS = 256 / VPR;
    const int h = blockIdx.y;
    const int row = blockIdx.x * ROWS + threadIdx.x / VPR;     // compressed row inside the head plane
    const int c0 = (threadIdx.x % VPR) * VEC;
    if (row >= total_c) return;
    const int seq = find_seq(map.cu_c, map.batch, row);
    if (row >= map.cu_c[map.batch]) return;                    // padding rows beyond the last sequence
    const int i = row - map.cu_c[seq];
    const T *src = k + (int64_t)map.cu[seq] * map.kv_tok_stride + (int64_t)h * map.kv_head_stride +
                   (int64_t)i * sc * map.kv_tok_stride + c0;
    float acc[VEC];
#pragma unroll
    for (int c = 0; c < VEC; ++c) acc[c] = 0.f;
    for (int u = 0; u < lc; ++u) {
        const T *r = src + (int64_t)u * map.kv_tok_stride;
#pragma unroll
        for (int c = 0; c < VEC; ++c) acc[c] += Elem<T>::load(r + c);
    }
    const float inv = 1.0f / (float)lc;
    float *dst = kc + ((int64_t)h * map.kc_total_c + row) * D + c0;
#pragma unroll
    for (int c = 0; c < VEC; ++c) dst[c] = acc[c] * inv;
}

template <typename T, int D>
static int launch_t(const Launch &L, const void *k, float *kc, int total_c) {
    constexpr int ROWS = 256 / (D / 8);
    dim3 grid((total_c + ROWS - 1) / ROWS, L.p->num_kv_heads);
    if (grid.x == 0) return INFLLMV2_OK;
    hipLaunchKernelGGL((compress_k_kernel<T, D>), grid, dim3(256), 0, L.stream, (const T *)k, L.map,
                       L.p->cmp_len, L.p->cmp_stride, total_c, kc);
    return hip_status(hipGetLastError());
}

// Compressed keys that became complete while a cached sequence grew from prev[b] to ctx[b] tokens: rows
// nc(prev[b]) .. nc(ctx[b]) - 1 of the pair's plane of the compressed-key cache.  One workgroup per new row.
template <typename T, int D>
__global__ void __launch_bounds__(D / 8)
compress_k_append_kernel(const T *__restrict__ k, int64_t kv_batch_stride, int64_t kv_head_stride, int64_t kv_tok_stride,
                         float *__restrict__ kc, int64_t kc_head_stride, const int32_t *__restrict__ prev,
                         const int32_t *__restrict__ ctx, int hkv, int lc, int sc) {
    const int pair = blockIdx.y, b = pair / hkv, h = pair - b * hkv;
    const int i = num_cmp(prev[b], lc, sc) + (int)blockIdx.x;
    if (i >= num_cmp(ctx[b], lc, sc)) return;
    const int c0 = threadIdx.x * 8;
    const T *src = k + (int64_t)b * kv_batch_stride + (int64_t)h * kv_head_stride + (int64_t)i * sc * kv_tok_stride + c0;
    float acc[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[c] = 0.f;
    for (int u = 0; u < lc; ++u) {
        const T *r = src + (int64_t)u * kv_tok_stride;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] += Elem<T>::load(r + c);
    }
    const float inv = 1.0f / (float)lc;
    float *dst = kc + (int64_t)pair * kc_head_stride + (int64_t)i * D + c0;
#pragma unroll
    for (int c = 0; c < 8; ++c) dst[c] = acc[c] * inv;
}

template <typename T, int D>
static int launch_append_t(const infllmv2_params *p, const void *k, int64_t bs, int64_t hs, int64_t ts, float *kc,
                           int64_t kc_head_stride, const int32_t *prev_d, const int32_t *ctx_d, int batch, int max_new,
                           hipStream_t stream) {
    hipLaunchKernelGGL((compress_k_append_kernel<T, D>), dim3(max_new, batch * p->num_kv_heads), dim3(D / 8), 0, stream,
                       (const T *)k, bs, hs, ts, kc, kc_head_stride, prev_d, ctx_d, p->num_kv_heads, p->cmp_len,
                       p->cmp_stride);
    return hip_status(hipGetLastError());
}

int launch_compress_k_append(const infllmv2_params *p, const void *k, int64_t bs, int64_t hs, int64_t ts, float *kc,
                             int64_t kc_head_stride, const int32_t *prev_d, const int32_t *ctx_d, int batch, int max_new,
                             hipStream_t stream) {
    const bool bf = p->dtype == INFLLMV2_BF16;
    if (p->head_dim == 128)
        return bf ? launch_append_t<bf16_t, 128>(p, k, bs, hs, ts, kc, kc_head_stride, prev_d, ctx_d, batch, max_new, stream)
                  : launch_append_t<float, 128>(p, k, bs, hs, ts, kc, kc_head_stride, prev_d, ctx_d, batch, max_new, stream);
    return bf ? launch_append_t<bf16_t, 64>(p, k, bs, hs, ts, kc, kc_head_stride, prev_d, ctx_d, batch, max_new, stream)
              : launch_append_t<float, 64>(p, k, bs, hs, ts, kc, kc_head_stride, prev_d, ctx_d, batch, max_new, stream);
}

int launch_compress_k(const Launch &L, const void *k, float *kc, int64_t total_c_rows) {
    const int tc = (int)total_c_rows;
    const bool bf = L.p->dtype == INFLLMV2_BF16;
    if (L.p->head_dim == 128) return bf ? launch_t<bf16_t, 128>(L, k, kc, tc) : launch_t<float, 128>(L, k, kc, tc);
    return bf ? launch_t<bf16_t, 64>(L, k, kc, tc) : launch_t<float, 64>(L, k, kc, tc);
}

}  // namespace ifv2
