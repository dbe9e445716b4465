// Stage 2: S^shared = sum over the GQA group of softmax(scale * Q K^{C1 T})  (Sec. 3.3 Eq. 4-5).
// Both kernels follow the two-pass scheme of Alg. 1 / Sec. 3.4: pass 1 finds the log-sum-exp of
// every (token, head) row on chip, pass 2 recomputes the logits, normalises, sums the G heads of
// the group on chip and stores only the group sum.  Per-head score rows never reach HBM.
#include "common.h"

namespace ifv2 {

// ------------------------------------------------------------------------------------------
// Generic fp32-arithmetic kernel: one workgroup per (query row, KV head); any G <= 16, d in {64,128},
// fp32 or bf16 inputs.  Used for fp32 data, unusual head shapes and single-row (decode) calls.
// ------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ void __launch_bounds__(256)
block_scores_generic(const T *__restrict__ q, const float *__restrict__ kc, RowMap map, int hq, int lc, int sc,
                     float scale, int dense_below, float *__restrict__ s_shared, int64_t row_stride) {
    const int row = blockIdx.x, h = blockIdx.y;
    const int G = hq / map.num_kv_heads;
    const RowLoc loc = locate(map, row);
    const int v = visible_cmp(loc.pos, lc, sc);
    if (v == 0 || loc.len < dense_below) return;      // dense sequences need no scores
    __shared__ float qs[kMaxGroup][D];
    __shared__ float red_m[4][kMaxGroup], red_l[4][kMaxGroup];
    __shared__ float lse_s[kMaxGroup];
    const int tid = threadIdx.x;
    for (int e = tid; e < kMaxGroup * D; e += 256) {
        int g = e / D, c = e % D;
        qs[g][c] = g < G ? Elem<T>::load(q + ((int64_t)row * hq + h * G + g) * D + c) * scale : 0.f;
    }
    __syncthreads();
    const float *kcb = kc_base(map, kc, loc.seq, h, D);
    float m[kMaxGroup], l[kMaxGroup];
#pragma unroll
    for (int g = 0; g < kMaxGroup; ++g) { m[g] = -INFINITY; l[g] = 0.f; }
    // pass 1: running (max, sum exp) per head, private to the thread
    for (int i = tid; i < v; i += 256) {
        float z[kMaxGroup];
#pragma unroll
        for (int g = 0; g < kMaxGroup; ++g) z[g] = 0.f;
        const float *kr = kcb + (int64_t)i * D;
        for (int c = 0; c < D; c += 4) {
            float4 kv = *reinterpret_cast<const float4 *>(kr + c);
#pragma unroll
            for (int g = 0; g < kMaxGroup; ++g)
                z[g] += qs[g][c] * kv.x + qs[g][c + 1] * kv.y + qs[g][c + 2] * kv.z + qs[g][c + 3] * kv.w;
        }
#pragma unroll
        for (int g = 0; g < kMaxGroup; ++g) {
            float mn = fmaxf(m[g], z[g]);
            l[g] = l[g] * __expf(m[g] - mn) + __expf(z[g] - mn);
            m[g] = mn;
        }
    }
    // merge across the workgroup
    const int lane = tid & 63, w = tid >> 6;
#pragma unroll
    for (int g = 0; g < kMaxGroup; ++g) {
        float mw = wave_max(m[g]);
        float lw = wave_sum(m[g] == -INFINITY ? 0.f : l[g] * __expf(m[g] - mw));
        if (lane == 0) { red_m[w][g] = mw; red_l[w][g] = lw; }
    }
    __syncthreads();
    if (tid < kMaxGroup) {
        float mm = fmaxf(fmaxf(red_m[0][tid], red_m[1][tid]), fmaxf(red_m[2][tid], red_m[3][tid]));
        float ll = 0.f;
        for (int k = 0; k < 4; ++k)
            if (red_m[k][tid] != -INFINITY) ll += red_l[k][tid] * __expf(red_m[k][tid] - mm);
        lse_s[tid] = mm + __logf(ll);
    }
    __syncthreads();
    // pass 2: recompute, normalise, sum the group
    float *out = s_shared + head_row(map, h, row) * row_stride;
    for (int i = tid; i < v; i += 256) {
        float z[kMaxGroup];
#pragma unroll
        for (int g = 0; g < kMaxGroup; ++g) z[g] = 0.f;
        const float *kr = kcb + (int64_t)i * D;
        for (int c = 0; c < D; c += 4) {
            float4 kv = *reinterpret_cast<const float4 *>(kr + c);
#pragma unroll
            for (int g = 0; g < kMaxGroup; ++g)
                z[g] += qs[g][c] * kv.x + qs[g][c + 1] * kv.y + qs[g][c + 2] * kv.z + qs[g][c + 3] * kv.w;
        }
        float s = 0.f;
#pragma unroll
        for (int g = 0; g < kMaxGroup; ++g)
            if (g < G) s += __expf(z[g] - lse_s[g]);
        out[i] = s;
    }
}

template <typename T, int D>
static int launch_generic(const Launch &L, const void *q, const float *kc, float *s_shared, int64_t row_stride) {
    dim3 grid(L.map.total_rows, L.p->num_kv_heads);
    if (grid.x == 0) return INFLLMV2_OK;
    hipLaunchKernelGGL((block_scores_generic<T, D>), grid, dim3(256), 0, L.stream, (const T *)q, kc, L.map,
                       L.p->num_q_heads, L.p->cmp_len, L.p->cmp_stride, L.p->softmax_scale, L.p->dense_threshold,
                       s_shared, row_stride);
    return hip_status(hipGetLastError());
}

int launch_block_scores(const Launch &L, const void *q, const float *kc, float *s_shared, int64_t row_stride) {
    const bool bf = L.p->dtype == INFLLMV2_BF16;
    if (L.p->head_dim == 128)
        return bf ? launch_generic<bf16_t, 128>(L, q, kc, s_shared, row_stride)
                  : launch_generic<float, 128>(L, q, kc, s_shared, row_stride);
    return bf ? launch_generic<bf16_t, 64>(L, q, kc, s_shared, row_stride)
              : launch_generic<float, 64>(L, q, kc, s_shared, row_stride);
}

}  // namespace ifv2
