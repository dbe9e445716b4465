// Stage 2: S^shared = sum over the GQA group of softmax(scale * Q K^{C1 T})  (Sec. 3.3 Eq. 4-5).
// Both kernels follow the two-pass scheme of Alg. 1 / Sec. 3.4: pass 1 finds the log-sum-exp of
// every (token, head) row on chip, pass 2 recomputes the logits, normalises, sums the G heads of
// the group on chip and stores only the group sum.  Per-head score rows never reach HBM.
#include <stdlib.h>

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


// ------------------------------------------------------------------------------------------
// MFMA kernel for bf16 Q, G = 16, d = 128 (the paper's head shape).
//
// A workgroup owns T consecutive tokens of one KV head; every wave keeps the Q rows of its TPW tokens in
// registers as MFMA A operands (M = the 16 heads of the group).  Compressed keys stream through LDS in
// tiles of 64 and each B fragment read from LDS is reused by all TPW tokens of the wave.  A lane then owns
// one key column and four heads, so
//   pass 1 keeps a private running (max, sum exp) per head with no cross-lane traffic in the loop, and
//   pass 2 sums its four heads in registers and finishes the head-group sum with a 3-step butterfly
//          across the four lane groups, after which the 64 lanes hold 64 consecutive keys' group sums.
// K^{C1} is float32 in HBM.  It is split on the way into LDS into a bf16 high part and a bf16 residual.
// Pass 1 (the normaliser, an average over many keys) uses the high part only; pass 2 adds the residual
// product so the stored scores carry ~16 mantissa bits of K^{C1} and selections do not flip on rounding.
// ------------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

namespace {

constexpr int SD = 128, SG = 16;
constexpr int SKS = SD + 8;                    // LDS row stride (bf16) of a compressed-key tile
constexpr int S_TILE = kBlock * SKS;           // one 64-key tile (hi or lo)
constexpr int S_STAGE = 2 * S_TILE;            // hi + lo
constexpr float S_LOG2E = 1.4426950408889634f;

struct ScoreArgs {
    const uint16_t *q;
    const float *kc;
    float *out;
    RowMap map;
    int hq, lc, sc, dense_below;
    float scale;
    int64_t row_stride;
};

template <int NW, int TPW, bool P1_LO>
struct ScoreKernel {
    static constexpr int T = NW * TPW;
    static constexpr int NTHR = NW * 64;
    static constexpr int NCH = 2048 / NTHR;        // float4 chunks of a 64 x 128 fp32 tile per thread

    __device__ static inline void load_tile(const float *kcb, int kt, int nc, int tid, float4 (&pf)[NCH]) {
#pragma unroll
        for (int r = 0; r < NCH; ++r) {
            const int c = tid + r * NTHR;
            const int row = kt * kBlock + (c >> 5), col = (c & 31) * 4;
            pf[r] = row < nc ? *reinterpret_cast<const float4 *>(kcb + (int64_t)row * SD + col)
                             : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    __device__ static inline void store_tile(uint16_t *stage, int tid, const float4 (&pf)[NCH]) {
#pragma unroll
        for (int r = 0; r < NCH; ++r) {
            const int c = tid + r * NTHR;
            const int row = c >> 5, col = (c & 31) * 4;
            const float x[4] = {pf[r].x, pf[r].y, pf[r].z, pf[r].w};
            uint16_t hi[4], lo[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                hi[e] = float_to_bf16(x[e]);
                lo[e] = float_to_bf16(x[e] - bf16_to_float(hi[e]));
            }
            uint2 h2, l2;
            h2.x = hi[0] | ((uint32_t)hi[1] << 16);
            h2.y = hi[2] | ((uint32_t)hi[3] << 16);
            l2.x = lo[0] | ((uint32_t)lo[1] << 16);
            l2.y = lo[2] | ((uint32_t)lo[3] << 16);
            *reinterpret_cast<uint2 *>(stage + row * SKS + col) = h2;
            *reinterpret_cast<uint2 *>(stage + S_TILE + row * SKS + col) = l2;
        }
    }

    // acc[i][nt] = Q_i (16 heads x 128) . kc_tile^T (128 x 16 keys of n-tile nt); B fragments shared by the tokens
    template <bool WITH_LO>
    __device__ static inline void tile_mma(const bf16x8 (&qf)[TPW][4], const uint16_t *stage, int lane,
                                           const bool (&active)[TPW], f32x4 (&acc)[TPW][4]) {
        const int n16 = lane & 15, g = lane >> 4;
        const uint16_t *bp = stage + n16 * SKS + g * 8;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) {
#pragma unroll
            for (int i = 0; i < TPW; ++i) acc[i][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const bf16x8 bh = *reinterpret_cast<const bf16x8 *>(bp + nt * 16 * SKS + ks * 32);
                bf16x8 bl;
                if (WITH_LO) bl = *reinterpret_cast<const bf16x8 *>(bp + S_TILE + nt * 16 * SKS + ks * 32);
#pragma unroll
                for (int i = 0; i < TPW; ++i) {
                    if (active[i]) {
                        acc[i][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[i][ks], bh, acc[i][nt], 0, 0, 0);
                        if (WITH_LO)
                            acc[i][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[i][ks], bl, acc[i][nt], 0, 0, 0);
                    }
                }
            }
        }
    }

    __device__ static void run(const ScoreArgs &a, int num_tiles) {
        extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
        __shared__ int s_seq, s_tile;
        const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
        const int h = blockIdx.y;
        const int tile_id = num_tiles - 1 - (int)blockIdx.x;     // longest rows first
        if (tid == 0) {
            int rem = tile_id, s = 0;
            for (; s < a.map.batch; ++s) {
                const int nt = (a.map.cu[s + 1] - a.map.cu[s] + T - 1) / T;
                if (rem < nt) break;
                rem -= nt;
            }
            s_seq = s;
            s_tile = rem;
        }
        __syncthreads();
        const int seq = s_seq;
        if (seq >= a.map.batch) return;
        const int tok0 = a.map.cu[seq], len = a.map.cu[seq + 1] - tok0;
        if (len < a.dense_below) return;
        const int t0 = s_tile * T;
        const int ntok = min(T, len - t0);
        const int nc = num_cmp(len, a.lc, a.sc);
        const int vis_last = min(visible_cmp(t0 + ntok - 1, a.lc, a.sc), nc);
        if (vis_last == 0) return;
        const int nkt = (vis_last + kBlock - 1) / kBlock;
        const int row0 = tok0 + t0;
        const float *kcb = a.kc + ((int64_t)h * a.map.kc_total_c + a.map.cu_c[seq]) * SD;
        const float c = a.scale * S_LOG2E;
        const int n16 = lane & 15, g = lane >> 4;

        bf16x8 qf[TPW][4];
        int vis[TPW];
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int ti = w * TPW + i;
            vis[i] = ti < ntok ? min(visible_cmp(t0 + ti, a.lc, a.sc), nc) : 0;
            const uint16_t *qp = a.q + ((int64_t)(row0 + ti) * a.hq + h * SG + n16) * SD + g * 8;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                uint4 raw = ti < ntok ? *reinterpret_cast<const uint4 *>(qp + ks * 32) : make_uint4(0, 0, 0, 0);
                qf[i][ks] = __builtin_bit_cast(bf16x8, raw);
            }
        }

        float4 pf[NCH];
        f32x4 acc[TPW][4];
        bool active[TPW];
        float m[TPW][4], l[TPW][4];
#pragma unroll
        for (int i = 0; i < TPW; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) { m[i][r] = -INFINITY; l[i][r] = 0.f; }

        // ------------------------------------------------ pass 1: log-sum-exp of every (token, head) row
        load_tile(kcb, 0, nc, tid, pf);
        store_tile(smem, tid, pf);
        __syncthreads();
        for (int kt = 0; kt < nkt; ++kt) {
            if (kt + 1 < nkt) load_tile(kcb, kt + 1, nc, tid, pf);
            const uint16_t *stage = smem + (kt & 1) * S_STAGE;
            const int kbase = kt * kBlock;
#pragma unroll
            for (int i = 0; i < TPW; ++i) active[i] = kbase < vis[i];
            if (P1_LO) tile_mma<true>(qf, stage, lane, active, acc);
            else tile_mma<false>(qf, stage, lane, active, acc);
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                if (!active[i]) continue;
                const bool edge = kbase + kBlock > vis[i];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float z[4];
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) {
                        z[nt] = acc[i][nt][r];
                        if (edge && kbase + nt * 16 + n16 >= vis[i]) z[nt] = -INFINITY;
                    }
                    const float mx = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
                    const float mn = fmaxf(m[i][r], mx);
                    const float ms = mn == -INFINITY ? 0.f : mn;
                    const float msc = ms * c;
                    float sum = l[i][r] * __builtin_amdgcn_exp2f((m[i][r] - ms) * c);
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) sum += __builtin_amdgcn_exp2f(z[nt] * c - msc);
                    l[i][r] = sum;
                    m[i][r] = mn;
                }
            }
            if (kt + 1 < nkt) store_tile(smem + ((kt + 1) & 1) * S_STAGE, tid, pf);
            __syncthreads();
        }
        // merge the 16 key lanes of each lane group; lse2 = log2 of the row's sum of 2^(c z)
        float lse2[TPW][4];
#pragma unroll
        for (int i = 0; i < TPW; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float mm = m[i][r], ll = l[i][r];
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) {
                    const float mo = __shfl_xor(mm, o), lo = __shfl_xor(ll, o);
                    const float mn = fmaxf(mm, mo);
                    const float ms = mn == -INFINITY ? 0.f : mn;
                    ll = ll * __builtin_amdgcn_exp2f((mm - ms) * c) + lo * __builtin_amdgcn_exp2f((mo - ms) * c);
                    mm = mn;
                }
                lse2[i][r] = mm * c + __log2f(ll);
            }

        // ------------------------------------------------ pass 2: normalised scores, group sum, store
        load_tile(kcb, 0, nc, tid, pf);
        store_tile(smem, tid, pf);
        __syncthreads();
        for (int kt = 0; kt < nkt; ++kt) {
            if (kt + 1 < nkt) load_tile(kcb, kt + 1, nc, tid, pf);
            const uint16_t *stage = smem + (kt & 1) * S_STAGE;
            const int kbase = kt * kBlock;
#pragma unroll
            for (int i = 0; i < TPW; ++i) active[i] = kbase < vis[i];
            tile_mma<true>(qf, stage, lane, active, acc);
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                if (!active[i]) continue;
                float s[4];
#pragma unroll
                for (int nt = 0; nt < 4; ++nt) {
                    float t = 0.f;
#pragma unroll
                    for (int r = 0; r < 4; ++r) t += __builtin_amdgcn_exp2f(acc[i][nt][r] * c - lse2[i][r]);
                    s[nt] = t;
                }
                // butterfly over the four lane groups: afterwards lane (n16, g) holds n-tile 2*(g&1) + (g>>1)
                const bool odd = g & 1, up = g & 2;
                const float a0 = (odd ? s[2] : s[0]) + __shfl_xor(odd ? s[0] : s[2], 16);
                const float a1 = (odd ? s[3] : s[1]) + __shfl_xor(odd ? s[1] : s[3], 16);
                const float f = (up ? a1 : a0) + __shfl_xor(up ? a0 : a1, 32);
                const int key = kbase + (2 * (g & 1) + (g >> 1)) * 16 + n16;
                if (key < vis[i])
                    a.out[((int64_t)h * a.map.total_rows + row0 + w * TPW + i) * a.row_stride + key] = f;
            }
            if (kt + 1 < nkt) store_tile(smem + ((kt + 1) & 1) * S_STAGE, tid, pf);
            __syncthreads();
        }
    }
};

template <int NW, int TPW, bool P1_LO>
__global__ void __launch_bounds__(NW * 64) block_scores_mfma_kernel(ScoreArgs a, int num_tiles) {
    ScoreKernel<NW, TPW, P1_LO>::run(a, num_tiles);
}

template <int NW, int TPW, bool P1_LO>
int launch_scores_mfma(const Launch &L, const ScoreArgs &a, const int32_t *cu_h) {
    constexpr int T = NW * TPW;
    int64_t tiles = 0;
    for (int s = 0; s < L.map.batch; ++s) tiles += (cu_h[s + 1] - cu_h[s] + T - 1) / T;
    if (tiles == 0) return INFLLMV2_OK;
    const size_t lds = (size_t)2 * S_STAGE * sizeof(uint16_t);
    auto kern = block_scores_mfma_kernel<NW, TPW, P1_LO>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return INFLLMV2_ERR_HIP;
    dim3 grid((unsigned)tiles, L.p->num_kv_heads);
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), lds, L.stream, a, (int)tiles);
    return hip_status(hipGetLastError());
}

}  // namespace

int launch_block_scores(const Launch &L, const void *q, const float *kc, float *s_shared, int64_t row_stride,
                        const int32_t *cu_h) {
    const bool bf = L.p->dtype == INFLLMV2_BF16;
    if (bf && cu_h != nullptr && L.map.ctx == nullptr && L.p->head_dim == SD &&
        L.p->num_q_heads / L.p->num_kv_heads == SG && (((uintptr_t)q | (uintptr_t)kc) & 15) == 0) {
        ScoreArgs a{(const uint16_t *)q, kc, s_shared, L.map, L.p->num_q_heads, L.p->cmp_len, L.p->cmp_stride,
                    L.p->dense_threshold, L.p->softmax_scale, row_stride};
        static const bool p1_hi_only = getenv("INFLLMV2_SCORES_P1_HI") != nullptr;   // experiment switch
        return p1_hi_only ? launch_scores_mfma<8, 4, false>(L, a, cu_h) : launch_scores_mfma<8, 4, true>(L, a, cu_h);
    }
    if (L.p->head_dim == 128)
        return bf ? launch_generic<bf16_t, 128>(L, q, kc, s_shared, row_stride)
                  : launch_generic<float, 128>(L, q, kc, s_shared, row_stride);
    return bf ? launch_generic<bf16_t, 64>(L, q, kc, s_shared, row_stride)
              : launch_generic<float, 64>(L, q, kc, s_shared, row_stride);
}

}  // namespace ifv2
