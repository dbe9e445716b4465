// Stage 4, generic fp32-arithmetic form: block-sparse causal attention over the selected blocks
// (Appendix Alg. 2) and dense causal attention (Eq. 1 / Appendix Alg. 3) for any G <= 16,
// d in {64, 128}, fp32 or bf16 data.  One workgroup per (query row, KV head); the G heads of the group
// share every K/V block it touches.  The bf16 G=16 d=128 shape has its own MFMA kernel; this one serves
// fp32 data, other head shapes and single-row (decode) calls.
#include "common.h"

namespace ifv2 {

template <typename T, int D>
__global__ void __launch_bounds__(256)
attn_generic_kernel(const T *__restrict__ q, const T *__restrict__ k, const T *__restrict__ v,
                    const int32_t *__restrict__ idx, int topk_total, int dense_below, RowMap map, int hq,
                    float scale, T *__restrict__ out, float *__restrict__ lse) {
    const int row = blockIdx.x, h = blockIdx.y;
    const int G = hq / map.num_kv_heads;
    const RowLoc loc = locate(map, row);
    const int t = loc.pos, bt = t / kBlock;
    const bool dense = idx == nullptr || loc.len < dense_below;
    const int32_t *my_idx = dense ? nullptr : idx + head_row(map, h, row) * topk_total;
    const int nsteps = dense ? bt + 1 : topk_total;

    __shared__ float qs[kMaxGroup][D];
    __shared__ float ps[kMaxGroup][kBlock];
    __shared__ float alpha_s[kMaxGroup];
    __shared__ float l_s[kMaxGroup], m_s[kMaxGroup];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    for (int e = tid; e < kMaxGroup * D; e += 256) {
        int g = e / D, c = e % D;
        qs[g][c] = g < G ? Elem<T>::load(q + ((int64_t)row * hq + h * G + g) * D + c) * scale : 0.f;
    }
    __syncthreads();
    const T *kb = k + loc.kv_base + (int64_t)h * map.kv_head_stride;
    const T *vb = v + loc.kv_base + (int64_t)h * map.kv_head_stride;

    constexpr int NACC = kMaxGroup * D / 256;      // outputs per thread (covers G = 16)
    float acc[NACC];
#pragma unroll
    for (int a = 0; a < NACC; ++a) acc[a] = 0.f;
    float m_run[4], l_run[4];                       // wave w owns heads w, w+4, w+8, w+12
#pragma unroll
    for (int a = 0; a < 4; ++a) { m_run[a] = -INFINITY; l_run[a] = 0.f; }

    for (int s = 0; s < nsteps; ++s) {
        const int j = dense ? s : my_idx[s];
        if (j < 0 || j > bt) continue;              // padding (or a block past the query): uniform skip
        const int u = j * kBlock + lane;            // this lane's key
        const bool valid = u <= t;                  // causal; also excludes keys past the sequence end
        // logits of heads w, w+4, ... for key `lane`
        float z[4] = {0.f, 0.f, 0.f, 0.f};
        if (valid) {
            const T *kr = kb + (int64_t)u * map.kv_tok_stride;
            for (int c = 0; c < D; ++c) {
                float kv = Elem<T>::load(kr + c);
#pragma unroll
                for (int a = 0; a < 4; ++a) z[a] += qs[w + 4 * a][c] * kv;
            }
        }
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int g = w + 4 * a;
            float zz = valid ? z[a] : -INFINITY;
            float mx = wave_max(zz);                // finite: key j*64 <= t is always valid
            float mn = fmaxf(m_run[a], mx);
            float pexp = valid ? __expf(zz - mn) : 0.f;
            float rs = wave_sum(pexp);
            float al = __expf(m_run[a] - mn);       // exp(-inf) = 0 on the first block
            l_run[a] = l_run[a] * al + rs;
            m_run[a] = mn;
            ps[g][lane] = pexp;
            if (lane == 0) alpha_s[g] = al;
        }
        __syncthreads();
        // O += P V for this thread's (head, channel) outputs
#pragma unroll
        for (int a = 0; a < NACC; ++a) {
            const int o = tid + a * 256;
            const int g = o / D, c = o % D;
            if (g < G) {
                float s_acc = 0.f;
                const int nkeys = min(kBlock, t - j * kBlock + 1);
                for (int kk = 0; kk < nkeys; ++kk)
                    s_acc += ps[g][kk] * Elem<T>::load(vb + (int64_t)(j * kBlock + kk) * map.kv_tok_stride + c);
                acc[a] = acc[a] * alpha_s[g] + s_acc;
            }
        }
        __syncthreads();
    }
    if (lane == 0) {
#pragma unroll
        for (int a = 0; a < 4; ++a) { l_s[w + 4 * a] = l_run[a]; m_s[w + 4 * a] = m_run[a]; }
    }
    __syncthreads();
#pragma unroll
    for (int a = 0; a < NACC; ++a) {
        const int o = tid + a * 256;
        const int g = o / D, c = o % D;
        if (g < G) Elem<T>::store(out + ((int64_t)row * hq + h * G + g) * D + c, acc[a] / l_s[g]);
    }
    if (lse != nullptr && tid < G) lse[qhead_row(map, h * G + tid, hq, row)] = m_s[tid] + __logf(l_s[tid]);
}

template <typename T, int D>
static int launch_t(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx,
                    int dense_below, void *out, float *lse) {
    dim3 grid(L.map.total_rows, L.p->num_kv_heads);
    if (grid.x == 0) return INFLLMV2_OK;
    hipLaunchKernelGGL((attn_generic_kernel<T, D>), grid, dim3(256), 0, L.stream, (const T *)q, (const T *)k,
                       (const T *)v, idx, L.p->topk_total, dense_below, L.map, L.p->num_q_heads,
                       L.p->softmax_scale, (T *)out, lse);
    return hip_status(hipGetLastError());
}

int launch_attn_generic(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx,
                        int dense_below, void *out, float *lse) {
    const bool bf = L.p->dtype == INFLLMV2_BF16;
    if (L.p->head_dim == 128)
        return bf ? launch_t<bf16_t, 128>(L, q, k, v, idx, dense_below, out, lse)
                  : launch_t<float, 128>(L, q, k, v, idx, dense_below, out, lse);
    return bf ? launch_t<bf16_t, 64>(L, q, k, v, idx, dense_below, out, lse)
              : launch_t<float, 64>(L, q, k, v, idx, dense_below, out, lse);
}

}  // namespace ifv2
