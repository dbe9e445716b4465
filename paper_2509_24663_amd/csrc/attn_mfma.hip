// Stage 4 on the matrix cores: block-sparse causal attention (Appendix Alg. 2) and dense causal attention
// (Eq. 1 / Appendix Alg. 3) for bf16 data with G = 16 query heads per KV head and d_h = 128.
//
// Alg. 2 gives every token a private pass over its selected K/V blocks.  Here a workgroup owns a tile of
// T consecutive tokens of one KV head instead: it forms the union of the tile's block lists, brings each
// K/V block of the union into LDS once, and every token that selected the block consumes it from there.
// Neighbouring tokens share most of their blocks (all init/local blocks, and most top-k blocks), so the
// gather traffic from L2 / HBM drops by the sharing factor while the arithmetic stays exactly the
// per-token softmax attention of Alg. 2.
//
// Per (token, block) the 16 heads of the group are one MFMA tile side: S^T = K_blk Q_t^T is computed as
// 4 key tiles x 4 k-steps of v_mfma_f32_16x16x32_bf16 (A = K rows from LDS, B = Q_t held in registers), so
// a lane owns one head and 16 keys: the running max / sum of the online softmax need two cross-lane steps,
// and P^T is already laid out as the B operand of O^T += V_blk^T P^T (A = V^T from LDS, 8 dim tiles x 2
// k-steps).  Keys are assigned to MFMA rows so that a lane's 8 probabilities of a k-step are 8 consecutive
// keys, which makes the V^T operand a single 16-byte LDS read.  V is transposed once per block while it
// is written to LDS.  Dense attention is the same kernel with "every block, every token".
#include "common.h"

namespace ifv2 {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

namespace {

constexpr int D = 128;            // head dim
constexpr int G = 16;             // heads per KV head
constexpr int KS = D + 8;         // LDS row stride of a K block, in bf16 (pad: conflict-free 16 B row reads)
constexpr int VS = kBlock + 8;    // LDS row stride of a transposed V block
constexpr int K_ELEMS = kBlock * KS;
constexpr int V_ELEMS = D * VS;
constexpr int STAGE_ELEMS = K_ELEMS + V_ELEMS;          // 17920 bf16 = 35840 B per stage
constexpr float LOG2E = 1.4426950408889634f;

struct AttnArgs {
    const uint16_t *q, *k, *v;
    const int32_t *idx;
    uint16_t *out;
    float *lse;
    RowMap map;
    int hq, topk_total, dense_below;
    float scale;
    int nb_cap;        // words reserved in LDS for the per-block token masks
    int list_cap;      // entries reserved for the union list
};

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int NW, int TPW>
struct TileKernel {
    static constexpr int T = NW * TPW;
    static constexpr int NTHR = NW * 64;
    static constexpr int KCH = 1024 / NTHR;      // 16-byte K chunks per thread per block
    static constexpr int VIT = 1024 / NTHR;      // (key quad, dim pair) V items per thread per block

    struct Prefetch {
        uint4 k[KCH];
        uint32_t v[VIT][4];
    };

    // ---- global -> registers for block j of the sequence (rows past the sequence end read as zero)
    __device__ static inline void load_block(const AttnArgs &a, const uint16_t *kb, const uint16_t *vb, int j, int len,
                                             int tid, Prefetch &pf) {
#pragma unroll
        for (int r = 0; r < KCH; ++r) {
            const int c = tid + r * NTHR;
            const int row = c >> 4, col = (c & 15) * 8;
            const int tok = j * kBlock + row;
            pf.k[r] = tok < len ? *reinterpret_cast<const uint4 *>(kb + (int64_t)tok * a.map.kv_tok_stride + col)
                                : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < VIT; ++r) {
            const int it = tid + r * NTHR;
            const int kq = it >> 6, dp = it & 63;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int tok = j * kBlock + kq * 4 + kk;
                pf.v[r][kk] = tok < len ? *reinterpret_cast<const uint32_t *>(vb + (int64_t)tok * a.map.kv_tok_stride + dp * 2)
                                        : 0u;
            }
        }
    }

    // ---- registers -> LDS stage: K row-major, V transposed ([dim][key])
    __device__ static inline void store_block(uint16_t *stage, int tid, const Prefetch &pf) {
        uint16_t *ks = stage, *vt = stage + K_ELEMS;
#pragma unroll
        for (int r = 0; r < KCH; ++r) {
            const int c = tid + r * NTHR;
            const int row = c >> 4, col = (c & 15) * 8;
            *reinterpret_cast<uint4 *>(ks + row * KS + col) = pf.k[r];
        }
#pragma unroll
        for (int r = 0; r < VIT; ++r) {
            const int it = tid + r * NTHR;
            const int kq = it >> 6, dp = it & 63;
            uint2 lo, hi;   // dim 2dp: low halves of the four keys; dim 2dp+1: high halves
            lo.x = (pf.v[r][0] & 0xffffu) | (pf.v[r][1] << 16);
            lo.y = (pf.v[r][2] & 0xffffu) | (pf.v[r][3] << 16);
            hi.x = (pf.v[r][0] >> 16) | (pf.v[r][1] & 0xffff0000u);
            hi.y = (pf.v[r][2] >> 16) | (pf.v[r][3] & 0xffff0000u);
            *reinterpret_cast<uint2 *>(vt + (2 * dp) * VS + kq * 4) = lo;
            *reinterpret_cast<uint2 *>(vt + (2 * dp + 1) * VS + kq * 4) = hi;
        }
    }

    struct TokState {
        bf16x8 qf[4];      // Q_t as MFMA B operand: head = lane % 16, dims ks*32 + (lane/16)*8 .. +8
        f32x4 o[8];        // O_t^T: dim tile dt, dims dt*16 + 4*(lane/16) + r, head = lane % 16
        float m, l;        // running max (raw logits) and this lane's share of the running sum
    };

    // ---- one (token, block) unit: S^T = K Q^T, online softmax, O^T += V^T P^T
    __device__ static inline void unit(TokState &st, const uint16_t *stage, int lane, bool diag, int key_limit, float c) {
        const int m16 = lane & 15, g = lane >> 4;
        const uint16_t *ks = stage + ((8 * (m16 >> 2) + (m16 & 3)) * KS + g * 8);
        const uint16_t *vt = stage + K_ELEMS + (m16 * VS + g * 8);
        f32x4 acc[4];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            acc[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(ks + (32 * (kt >> 1) + 4 * (kt & 1)) * KS + s * 32);
                acc[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, st.qf[s], acc[kt], 0, 0, 0);
            }
        }
        if (diag) {   // keys after the query token are masked
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int key = 32 * (kt >> 1) + 8 * g + 4 * (kt & 1) + r;
                    if (key > key_limit) acc[kt][r] = -INFINITY;
                }
        }
        float mx = acc[0][0];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r) mx = fmaxf(mx, acc[kt][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(st.m, mx);
        const float alpha = fast_exp2((st.m - m_new) * c);
        const float mc = m_new * c;
        st.m = m_new;
        float ls = 0.f;
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                acc[kt][r] = fast_exp2(acc[kt][r] * c - mc);
                ls += acc[kt][r];
            }
        st.l = st.l * alpha + ls;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) st.o[dt] *= alpha;
        bf16x8 pb[2];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                pb[s][r] = (__bf16)acc[2 * s][r];
                pb[s][4 + r] = (__bf16)acc[2 * s + 1][r];
            }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(vt + dt * 16 * VS + s * 32);
                st.o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[s], st.o[dt], 0, 0, 0);
            }
    }

    __device__ static void run(const AttnArgs &a, int num_tiles) {
        extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
        uint16_t *stages = smem;
        uint32_t *masks = reinterpret_cast<uint32_t *>(smem + 2 * STAGE_ELEMS);
        int32_t *list_j = reinterpret_cast<int32_t *>(masks + a.nb_cap);
        __shared__ int s_seq, s_tile, s_ne;

        const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
        const int h = blockIdx.y;
        const int tile_id = num_tiles - 1 - (int)blockIdx.x;     // late (long-context) tiles first
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
        const int t0 = s_tile * T;                       // first token of the tile (position in the sequence)
        const int ntok = min(T, len - t0);
        const int bt = t0 / kBlock, nblk = bt + 1;       // T divides 64: the tile lies in one block
        const bool dense = a.idx == nullptr || len < a.dense_below;
        const int row0 = tok0 + t0;                      // packed row of the tile's first token
        const uint16_t *kb = a.k + (int64_t)tok0 * a.map.kv_tok_stride + (int64_t)h * a.map.kv_head_stride;
        const uint16_t *vb = a.v + (int64_t)tok0 * a.map.kv_tok_stride + (int64_t)h * a.map.kv_head_stride;

        // ---- union of the tile's block lists: masks[j] has bit ti set if token ti selected block j
        int ne;
        if (!dense) {
            for (int j = tid; j < nblk; j += NTHR) masks[j] = 0u;
            __syncthreads();
            const int tk = a.topk_total;
            for (int e = tid; e < ntok * tk; e += NTHR) {
                const int ti = e / tk;
                const int j = a.idx[((int64_t)h * a.map.total_rows + row0 + ti) * tk + (e - ti * tk)];
                if (j >= 0 && j <= bt) atomicOr(&masks[j], 1u << ti);
            }
            __syncthreads();
            if (w == 0) {
                int base = 0;
                for (int cbase = 0; cbase < nblk; cbase += 64) {
                    const int j = cbase + lane;
                    const uint32_t mk = j < nblk ? masks[j] : 0u;
                    const uint64_t b = __ballot(mk != 0u);
                    if (mk != 0u) list_j[base + __popcll(b & ((1ull << lane) - 1ull))] = j;
                    base += __popcll(b);
                }
                if (lane == 0) s_ne = base;
            }
            __syncthreads();
            ne = s_ne;
        } else {
            ne = nblk;
        }

        // ---- this wave's tokens: ti = i * NW + w (interleaved so the waves' loads stay similar)
        TokState st[TPW];
        const int m16 = lane & 15, g = lane >> 4;
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int ti = i * NW + w;
            const uint16_t *qp = a.q + ((int64_t)(row0 + ti) * a.hq + h * G + m16) * D + g * 8;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                uint4 raw = ti < ntok ? *reinterpret_cast<const uint4 *>(qp + s * 32) : make_uint4(0, 0, 0, 0);
                st[i].qf[s] = __builtin_bit_cast(bf16x8, raw);
            }
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) st[i].o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
            st[i].m = -INFINITY;
            st[i].l = 0.f;
        }
        const float c = a.scale * LOG2E;
        const uint32_t full = ntok >= 32 ? 0xffffffffu : ((1u << ntok) - 1u);

        Prefetch pf;
        if (ne > 0) {
            load_block(a, kb, vb, dense ? 0 : list_j[0], len, tid, pf);
            store_block(stages, tid, pf);
        }
        __syncthreads();
        for (int e = 0; e < ne; ++e) {
            const int j = dense ? e : list_j[e];
            const uint32_t mk = dense ? full : masks[j];
            if (e + 1 < ne) load_block(a, kb, vb, dense ? e + 1 : list_j[e + 1], len, tid, pf);
            const uint16_t *stage = stages + (e & 1) * STAGE_ELEMS;
            const bool diag = j == bt;
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int ti = i * NW + w;
                if (mk & (1u << ti)) unit(st[i], stage, lane, diag, t0 + ti - j * kBlock, c);
            }
            if (e + 1 < ne) store_block(stages + ((e + 1) & 1) * STAGE_ELEMS, tid, pf);
            __syncthreads();
        }

        // ---- normalise and store
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int ti = i * NW + w;
            if (ti >= ntok) continue;
            float l = st[i].l;
            l += __shfl_xor(l, 16);
            l += __shfl_xor(l, 32);
            const float inv = l > 0.f ? 1.0f / l : 0.f;
            uint16_t *op = a.out + ((int64_t)(row0 + ti) * a.hq + h * G + m16) * D + g * 4;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                uint2 pk;
                pk.x = (uint32_t)float_to_bf16(st[i].o[dt][0] * inv) | ((uint32_t)float_to_bf16(st[i].o[dt][1] * inv) << 16);
                pk.y = (uint32_t)float_to_bf16(st[i].o[dt][2] * inv) | ((uint32_t)float_to_bf16(st[i].o[dt][3] * inv) << 16);
                *reinterpret_cast<uint2 *>(op + dt * 16) = pk;
            }
            if (a.lse != nullptr && g == 0)
                a.lse[(int64_t)(h * G + m16) * a.map.total_rows + row0 + ti] = st[i].m * a.scale + __logf(l);
        }
    }
};

template <int NW, int TPW>
__global__ void __launch_bounds__(NW * 64) attn_tile_kernel(AttnArgs a, int num_tiles) {
    TileKernel<NW, TPW>::run(a, num_tiles);
}

template <int NW, int TPW>
int launch_tile(const Launch &L, const AttnArgs &a0, const int32_t *cu_h) {
    constexpr int T = NW * TPW;
    AttnArgs a = a0;
    int64_t tiles = 0;
    for (int s = 0; s < L.map.batch; ++s) tiles += (cu_h[s + 1] - cu_h[s] + T - 1) / T;
    if (tiles == 0) return INFLLMV2_OK;
    const int nb_max = (L.max_len + kBlock - 1) / kBlock;
    a.nb_cap = a.idx ? (nb_max + 3) / 4 * 4 : 0;
    a.list_cap = a.idx ? min(nb_max, T * L.p->topk_total) : 0;
    const size_t lds = (size_t)2 * STAGE_ELEMS * sizeof(uint16_t) + (size_t)(a.nb_cap + a.list_cap) * 4;
    if (lds > 160 * 1024) return INFLLMV2_ERR_UNSUPPORTED;      // > ~2.8M tokens per sequence
    auto kern = attn_tile_kernel<NW, TPW>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return INFLLMV2_ERR_HIP;
    }
    dim3 grid((unsigned)tiles, L.p->num_kv_heads);
    hipLaunchKernelGGL(kern, grid, dim3(NW * 64), lds, L.stream, a, (int)tiles);
    return hip_status(hipGetLastError());
}

}  // namespace

bool attn_mfma_supported(const infllmv2_params *p) {
    return p->dtype == INFLLMV2_BF16 && p->head_dim == D && p->num_q_heads / p->num_kv_heads == G;
}

int launch_attn_mfma(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx,
                     int dense_below, void *out, float *lse, const int32_t *cu_h) {
    // 16-byte vector loads need 8-element aligned strides
    if (L.map.kv_tok_stride % 8 != 0 || L.map.kv_head_stride % 8 != 0) return INFLLMV2_ERR_UNSUPPORTED;
    AttnArgs a;
    a.q = (const uint16_t *)q;
    a.k = (const uint16_t *)k;
    a.v = (const uint16_t *)v;
    a.idx = idx;
    a.out = (uint16_t *)out;
    a.lse = lse;
    a.map = L.map;
    a.hq = L.p->num_q_heads;
    a.topk_total = L.p->topk_total;
    a.dense_below = dense_below;
    a.scale = L.p->softmax_scale;
    a.nb_cap = a.list_cap = 0;
    return launch_tile<4, 4>(L, a, cu_h);
}

}  // namespace ifv2
