// Gradients of stage 4 -- block-sparse causal attention over a given selection (Appendix Alg. 2), or dense causal
// attention (Eq. 1) -- with respect to Q, K and V.  The selection of stages 1-3 only picks blocks (Sec. 3.3), so it
// carries no gradient and is an input here.  The paper gives no backward algorithm; this is the chain rule on
// O = softmax(z) V, z = scale * q k^T, using the log-sum-exp the forward pass stored (Alg. 2 keeps it for this):
//     p_u  = exp(z_u - lse)                     dp_u = <dO, v_u>             Delta = <dO, O> (= sum_u p_u dp_u)
//     dz_u = p_u (dp_u - Delta)                 dq   = scale * sum_u dz_u k_u
//     dk_u += scale * dz_u q                    dv_u += p_u dO               (summed over rows and over the group)
// This file: fp32 arithmetic on the vector units for any G <= 16, d in {64, 128}, fp32 or bf16 data (the paper's
// head shape in bf16 takes the matrix-core path of attn_bwd_mfma.hip instead), in three kernels:
//   delta : Delta per (row, query head)
//   dq    : one workgroup per (row, KV head), the loop of the forward generic kernel
//   dkv   : one workgroup per (KV block, chunk of 256 later tokens, KV head): finds the tokens of its chunk that
//           selected the block, accumulates the block's 64 rows of dK and dV in registers and adds them to the
//           float32 result with atomics (one add per element and workgroup; the order of the adds, and with it the
//           last bits of dK and dV, can differ from run to run).
#include <algorithm>

#include "common.h"

namespace ifv2 {

namespace {

constexpr int BWD_CHUNK = 256;      // tokens per dkv workgroup

template <typename T>
struct BwdArgs {
    const T *q, *k, *v, *out, *dout;
    const float *lse;
    const int32_t *idx;         // nullptr: dense
    int topk_total, dense_below, hq;
    float scale;
    RowMap map;
    float *delta;               // [hq, T] scratch
    T *dq;
    float *dk, *dv;             // [hkv, T, D]
};

template <typename T, int D>
__global__ void __launch_bounds__(256) bwd_delta_kernel(BwdArgs<T> a) {
    // one wave per (row, query head)
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (item >= (int64_t)a.map.total_rows * a.hq) return;
    const int row = (int)(item / a.hq), qh = (int)(item % a.hq);
    const T *o = a.out + ((int64_t)row * a.hq + qh) * D, *g = a.dout + ((int64_t)row * a.hq + qh) * D;
    float s = 0.f;
    for (int c = lane; c < D; c += 64) s += Elem<T>::load(o + c) * Elem<T>::load(g + c);
    s = wave_sum(s);
    if (lane == 0) a.delta[qhead_row(a.map, qh, a.hq, row)] = s;
}

template <typename T, int D>
__global__ void __launch_bounds__(256) bwd_dq_kernel(BwdArgs<T> a) {
    const int row = blockIdx.x, h = blockIdx.y;
    const int G = a.hq / a.map.num_kv_heads;
    const RowLoc loc = locate(a.map, row);
    const int t = loc.pos, bt = t / kBlock;
    const bool dense = a.idx == nullptr || loc.len < a.dense_below;
    const int32_t *my_idx = dense ? nullptr : a.idx + head_row(a.map, h, row) * a.topk_total;
    const int nsteps = dense ? bt + 1 : a.topk_total;

    __shared__ float qs[kMaxGroup][D], gs[kMaxGroup][D];      // scale * q, dO
    __shared__ float dzs[kMaxGroup][kBlock];
    __shared__ float lse_s[kMaxGroup], delta_s[kMaxGroup];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    for (int e = tid; e < kMaxGroup * D; e += 256) {
        const int g = e / D, c = e % D;
        const int64_t off = ((int64_t)row * a.hq + h * G + g) * D + c;
        qs[g][c] = g < G ? Elem<T>::load(a.q + off) * a.scale : 0.f;
        gs[g][c] = g < G ? Elem<T>::load(a.dout + off) : 0.f;
    }
    if (tid < kMaxGroup) {
        lse_s[tid] = tid < G ? a.lse[qhead_row(a.map, h * G + tid, a.hq, row)] : 0.f;
        delta_s[tid] = tid < G ? a.delta[qhead_row(a.map, h * G + tid, a.hq, row)] : 0.f;
    }
    __syncthreads();
    const T *kb = a.k + loc.kv_base + (int64_t)h * a.map.kv_head_stride;
    const T *vb = a.v + loc.kv_base + (int64_t)h * a.map.kv_head_stride;
    constexpr int NACC = kMaxGroup * D / 256;
    float acc[NACC];
#pragma unroll
    for (int x = 0; x < NACC; ++x) acc[x] = 0.f;

    for (int s = 0; s < nsteps; ++s) {
        const int j = dense ? s : my_idx[s];
        if (j < 0 || j > bt) continue;
        const int u = j * kBlock + lane;
        const bool valid = u <= t;
        float z[4] = {0.f, 0.f, 0.f, 0.f}, dp[4] = {0.f, 0.f, 0.f, 0.f};     // heads w, w+4, w+8, w+12
        if (valid) {
            const T *kr = kb + (int64_t)u * a.map.kv_tok_stride, *vr = vb + (int64_t)u * a.map.kv_tok_stride;
            for (int c = 0; c < D; ++c) {
                const float kv = Elem<T>::load(kr + c), vv = Elem<T>::load(vr + c);
#pragma unroll
                for (int x = 0; x < 4; ++x) {
                    z[x] += qs[w + 4 * x][c] * kv;
                    dp[x] += gs[w + 4 * x][c] * vv;
                }
            }
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int g = w + 4 * x;
            const float p = valid ? __expf(z[x] - lse_s[g]) : 0.f;
            dzs[g][lane] = p * (dp[x] - delta_s[g]);
        }
        __syncthreads();
        const int nkeys = min(kBlock, t - j * kBlock + 1);
#pragma unroll
        for (int x = 0; x < NACC; ++x) {
            const int o = tid + x * 256;
            const int g = o / D, c = o % D;
            if (g < G) {
                float sacc = 0.f;
                for (int kk = 0; kk < nkeys; ++kk)
                    sacc += dzs[g][kk] * Elem<T>::load(kb + (int64_t)(j * kBlock + kk) * a.map.kv_tok_stride + c);
                acc[x] += sacc;
            }
        }
        __syncthreads();
    }
#pragma unroll
    for (int x = 0; x < NACC; ++x) {
        const int o = tid + x * 256;
        const int g = o / D, c = o % D;
        if (g < G) Elem<T>::store(a.dq + ((int64_t)row * a.hq + h * G + g) * D + c, acc[x] * a.scale);
    }
}

// is block j in the ascending, -1 padded list e[0 .. n)?
__device__ inline bool list_has(const int32_t *e, int n, int j) {
    int lo = 0, hi = n;                      // first position whose entry is >= j (padding counts as +inf)
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        const int x = e[mid];
        if (x >= 0 && x < j) lo = mid + 1; else hi = mid;
    }
    return lo < n && e[lo] == j;
}

template <typename T, int D>
__global__ void __launch_bounds__(256) bwd_dkv_kernel(BwdArgs<T> a, int num_blocks) {
    extern __shared__ float lds[];
    constexpr int DS = D + 1;                                  // padded row: lanes read different rows
    float *ks = lds, *vs = lds + kBlock * DS;                  // the block's K and V rows
    float *qs = vs + kBlock * DS, *gs = qs + kMaxGroup * D;     // scale * q, dO of the current token
    float *ps = gs + kMaxGroup * D, *dzs = ps + kMaxGroup * kBlock;
    __shared__ int s_seq, s_j, s_list[BWD_CHUNK], s_wave_cnt[4];
    __shared__ float lse_s[kMaxGroup], delta_s[kMaxGroup];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int h = blockIdx.z, G = a.hq / a.map.num_kv_heads;
    if (tid == 0) {
        int rem = blockIdx.y, s = 0;
        for (; s < a.map.batch; ++s) {
            const int nb = (a.map.cu[s + 1] - a.map.cu[s] + kBlock - 1) / kBlock;
            if (rem < nb) break;
            rem -= nb;
        }
        s_seq = s;
        s_j = rem;
    }
    __syncthreads();
    const int seq = s_seq, j = s_j;
    if (seq >= a.map.batch) return;
    const int tok0 = a.map.cu[seq], len = a.map.cu[seq + 1] - tok0;
    // tokens of this chunk that can see the block: [max(chunk start, 64 j), min(chunk end, len))
    const int c0 = blockIdx.x * BWD_CHUNK, c1 = min(c0 + BWD_CHUNK, len);
    if (c1 <= j * kBlock || c0 >= len) return;
    const bool dense = a.idx == nullptr || len < a.dense_below;

    // ---- which tokens of the chunk selected the block (in token order)
    const int t_mine = c0 + tid;
    bool sel = t_mine < c1 && t_mine >= j * kBlock;
    if (sel && !dense) sel = list_has(a.idx + head_row(a.map, h, tok0 + t_mine) * a.topk_total, a.topk_total, j);
    const uint64_t bal = __ballot(sel);
    if (lane == 0) s_wave_cnt[w] = __popcll(bal);
    __syncthreads();
    int base = 0, total = 0;
    for (int x = 0; x < 4; ++x) {
        if (x < w) base += s_wave_cnt[x];
        total += s_wave_cnt[x];
    }
    if (sel) s_list[base + __popcll(bal & ((1ull << lane) - 1ull))] = t_mine;
    if (total == 0) return;

    // ---- the block's K and V rows (zero past the end of the sequence)
    const int64_t kv_base = (int64_t)tok0 * a.map.kv_tok_stride + (int64_t)h * a.map.kv_head_stride;
    for (int e = tid; e < kBlock * D; e += 256) {
        const int r = e / D, c = e % D, u = j * kBlock + r;
        const int64_t off = kv_base + (int64_t)u * a.map.kv_tok_stride + c;
        ks[r * DS + c] = u < len ? Elem<T>::load(a.k + off) : 0.f;
        vs[r * DS + c] = u < len ? Elem<T>::load(a.v + off) : 0.f;
    }
    // this thread accumulates key `lane`, channels w * D/4 .. + D/4
    constexpr int NC = D / 4;
    float acc_k[NC], acc_v[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) acc_k[c] = acc_v[c] = 0.f;
    __syncthreads();

    for (int it = 0; it < total; ++it) {
        const int t = s_list[it], row = tok0 + t;
        for (int e = tid; e < kMaxGroup * D; e += 256) {
            const int g = e / D, c = e % D;
            const int64_t off = ((int64_t)row * a.hq + h * G + g) * D + c;
            qs[e] = g < G ? Elem<T>::load(a.q + off) * a.scale : 0.f;
            gs[e] = g < G ? Elem<T>::load(a.dout + off) : 0.f;
        }
        if (tid < kMaxGroup) {
            lse_s[tid] = tid < G ? a.lse[qhead_row(a.map, h * G + tid, a.hq, row)] : 0.f;
            delta_s[tid] = tid < G ? a.delta[qhead_row(a.map, h * G + tid, a.hq, row)] : 0.f;
        }
        __syncthreads();
        const bool valid = j * kBlock + lane <= t;             // causal (t < len, so also inside the sequence)
        float z[4] = {0.f, 0.f, 0.f, 0.f}, dp[4] = {0.f, 0.f, 0.f, 0.f};     // heads w, w+4, w+8, w+12 of key `lane`
        for (int c = 0; c < D; ++c) {
            const float kv = ks[lane * DS + c], vv = vs[lane * DS + c];
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                z[x] += qs[(w + 4 * x) * D + c] * kv;
                dp[x] += gs[(w + 4 * x) * D + c] * vv;
            }
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int g = w + 4 * x;
            const float p = valid && g < G ? __expf(z[x] - lse_s[g]) : 0.f;
            ps[g * kBlock + lane] = p;
            dzs[g * kBlock + lane] = p * (dp[x] - delta_s[g]);
        }
        __syncthreads();
        for (int g = 0; g < G; ++g) {
            const float p = ps[g * kBlock + lane], dz = dzs[g * kBlock + lane];
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                acc_v[c] += p * gs[g * D + w * NC + c];
                acc_k[c] += dz * qs[g * D + w * NC + c];        // qs carries the scale
            }
        }
        __syncthreads();
    }
    const int u = j * kBlock + lane;
    if (u < len) {
        float *dk = a.dk + ((int64_t)h * a.map.total_rows + tok0 + u) * D + w * NC;
        float *dv = a.dv + ((int64_t)h * a.map.total_rows + tok0 + u) * D + w * NC;
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            atomicAdd(dk + c, acc_k[c]);
            atomicAdd(dv + c, acc_v[c]);
        }
    }
}

__global__ void __launch_bounds__(256) bwd_zero_kernel(float4 *p, int64_t n4) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256)
        p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

template <typename T, int D>
int launch_t(const Launch &L, BwdArgs<T> a, const int32_t *cu_h) {
    const int64_t rows = L.map.total_rows;
    if (rows == 0) return INFLLMV2_OK;
    int64_t nblocks = 0;
    for (int s = 0; s < L.map.batch; ++s) nblocks += (cu_h[s + 1] - cu_h[s] + kBlock - 1) / kBlock;
    const int hkv = L.p->num_kv_heads;
    if (nblocks > 65535 || hkv > 65535) return INFLLMV2_ERR_UNSUPPORTED;      // grid.y / grid.z limits
    void *ws = L.ws;         // <dO, O> per (row, head)
    if (ws == nullptr || L.ws_bytes < (size_t)rows * a.hq * sizeof(float)) return INFLLMV2_ERR_WORKSPACE_TOO_SMALL;
    a.delta = (float *)ws;
    const int64_t n4 = rows * hkv * D / 4;
    hipLaunchKernelGGL(bwd_zero_kernel, dim3((unsigned)std::min<int64_t>((n4 + 255) / 256, 4096)), dim3(256), 0, L.stream,
                       (float4 *)a.dk, n4);
    hipLaunchKernelGGL(bwd_zero_kernel, dim3((unsigned)std::min<int64_t>((n4 + 255) / 256, 4096)), dim3(256), 0, L.stream,
                       (float4 *)a.dv, n4);
    hipLaunchKernelGGL((bwd_delta_kernel<T, D>), dim3((unsigned)((rows * a.hq + 3) / 4)), dim3(256), 0, L.stream, a);
    hipLaunchKernelGGL((bwd_dq_kernel<T, D>), dim3((unsigned)rows, hkv), dim3(256), 0, L.stream, a);
    const size_t lds = ((size_t)2 * kBlock * (D + 1) + 2 * kMaxGroup * D + 2 * kMaxGroup * kBlock) * sizeof(float);
    auto kern = bwd_dkv_kernel<T, D>;
    hipError_t e = hipSuccess;
    if (lds > 48 * 1024)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) {
        const unsigned chunks = (unsigned)((L.max_len + BWD_CHUNK - 1) / BWD_CHUNK);
        hipLaunchKernelGGL(kern, dim3(chunks, (unsigned)nblocks, hkv), dim3(256), lds, L.stream, a, (int)nblocks);
        e = hipGetLastError();
    }
    return hip_status(e);
}

template <typename T>
int launch_d(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx, int dense_below,
             const void *out, const float *lse, const void *dout, void *dq, float *dk, float *dv, const int32_t *cu_h) {
    BwdArgs<T> a{(const T *)q, (const T *)k, (const T *)v, (const T *)out, (const T *)dout, lse, idx,
                 L.p->topk_total, dense_below, L.p->num_q_heads, L.p->softmax_scale, L.map, nullptr, (T *)dq, dk, dv};
    return L.p->head_dim == 128 ? launch_t<T, 128>(L, a, cu_h) : launch_t<T, 64>(L, a, cu_h);
}

}  // namespace

// matrix-core path for the paper's head shape (attn_bwd_mfma.hip); INFLLMV2_ERR_UNSUPPORTED = not covered
int launch_attn_bwd_mfma(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx,
                         int dense_below, const void *out, const float *lse, const void *dout, void *dq, float *dk,
                         float *dv, const int32_t *cu_h);

bool bwd_mfma_params(const infllmv2_params *p);
size_t bwd_mfma_ws_bytes(const infllmv2_params *p, const BatchTotals &t, bool with_bitmap);

size_t attn_bwd_ws_bytes(const infllmv2_params *p, const BatchTotals &t, bool with_bitmap) {
    // (a call whose pointers or strides rule out the matrix-core path needs less: the bound still holds)
    if (bwd_mfma_params(p)) return bwd_mfma_ws_bytes(p, t, with_bitmap);
    return align256((size_t)t.rows * p->num_q_heads * sizeof(float));
}

int launch_attn_bwd(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx, int dense_below,
                    const void *out, const float *lse, const void *dout, void *dq, float *dk, float *dv,
                    const int32_t *cu_h) {
    const int st = launch_attn_bwd_mfma(L, q, k, v, idx, dense_below, out, lse, dout, dq, dk, dv, cu_h);
    if (st != INFLLMV2_ERR_UNSUPPORTED) return st;
    return L.p->dtype == INFLLMV2_BF16
               ? launch_d<bf16_t>(L, q, k, v, idx, dense_below, out, lse, dout, dq, dk, dv, cu_h)
               : launch_d<float>(L, q, k, v, idx, dense_below, out, lse, dout, dq, dk, dv, cu_h);
}

}  // namespace ifv2
