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
// Data movement: K and V blocks go from global memory straight into LDS (global_load_lds, 16 bytes per
// lane, no register staging), row-major, with the 16-byte chunks of a row XOR-swizzled by the row number
// so that both operand reads below are spread over all banks.
//
// Per (token, block) the 16 heads of the group are one MFMA tile side.  S^T = K_blk Q_t^T is 4 key tiles x
// 4 k-steps of v_mfma_f32_16x16x32_bf16 (A = K rows from LDS, B = Q_t held in registers), so a lane owns
// one head and 16 keys: the online softmax needs two cross-lane steps for the row max and none for the row
// sum (kept as per-lane partial sums until the end).  P^T is then already laid out as the B operand of
// O^T += V_blk^T P^T (8 dim tiles x 2 k-steps); its A operand V^T is read from the row-major V block with
// the transposing LDS read (ds_read_b64_tr_b16), two reads per operand.  Dense attention is the same
// kernel with "every block, every token".
#include <stdlib.h>
#include <string.h>

#include "common.h"

namespace ifv2 {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));

namespace {

constexpr int D = 128;            // head dim
constexpr int G = 16;             // heads per KV head
constexpr int TILE_ELEMS = kBlock * D;            // one K or V block in LDS: 64 rows x 256 B, unpadded
constexpr int STAGE_ELEMS = 2 * TILE_ELEMS;       // K then V: 32 KB per stage
constexpr float LOG2E = 1.4426950408889634f;
constexpr int WAIT_VMCNT0 = 0x0F70;               // s_waitcnt vmcnt(0), other counters untouched

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

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

template <int NW, int TPW>
struct TileKernel {
    static constexpr int T = NW * TPW;
    static constexpr int NTHR = NW * 64;
    static_assert(32 % NW == 0 || NW == 32, "32 one-KB load instructions are dealt round-robin to the waves");

    // ---- block j of the sequence: global -> LDS stage, asynchronously.  One instruction moves 1 KB = 4 rows;
    // lane l fills LDS slot (row 4q + l/16, physical chunk l%16), which holds logical chunk (l%16) ^ (row%16).
    // Rows past the end of the sequence re-read the last valid row (finite data, always masked by causality).
    __device__ static inline void issue_block_load(const AttnArgs &a, const uint16_t *kb, const uint16_t *vb, int j,
                                                   int len, uint16_t *stage, int w, int lane) {
#pragma unroll
        for (int qi = w; qi < 32; qi += NW) {
            const int q16 = qi & 15;                       // 16 instructions per tile
            const int row = 4 * q16 + (lane >> 4);
            const int chunk = (lane & 15) ^ (row & 15);
            const int tok = min(j * kBlock + row, len - 1);
            const uint16_t *src = (qi < 16 ? kb : vb) + (int64_t)tok * a.map.kv_tok_stride + chunk * 8;
            uint16_t *dst = stage + (qi < 16 ? 0 : TILE_ELEMS) + q16 * 512;
            __builtin_amdgcn_global_load_lds((glb_void *)src, (lds_void *)dst, 16, 0, 0);
        }
    }

    struct TokState {
        bf16x8 qf[4];      // Q_t as MFMA B operand: head = lane % 16, dims ks*32 + (lane/16)*8 .. +8
        f32x4 o[8];        // O_t^T: dim tile dt, dims dt*16 + 4*(lane/16) + r, head = lane % 16
        float m, l;        // running max (raw logits) and this lane's share of the running sum
    };

    struct LaneOffs {
        int kx[4];         // K operand: element offset of (row m16, logical chunk 4s+g) in a swizzled tile
        int vx[8];         // V operand source address of this lane for dim tile dt (transposing read)
    };

    __device__ static inline LaneOffs lane_offsets(int lane) {
        LaneOffs o;
        const int m16 = lane & 15, g = lane >> 4;
#pragma unroll
        for (int s = 0; s < 4; ++s) o.kx[s] = m16 * D + (((4 * s + g) ^ m16) << 3);
        // transposing read: within a group of 16 lanes, lane L supplies 4 consecutive dims of key row L/4 and
        // receives, for its dim (= L), the values of 4 consecutive key rows.
        const int rowlow = 4 * g + (m16 >> 2);
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            o.vx[dt] = rowlow * D + (((2 * dt + ((m16 >> 1) & 1)) ^ rowlow) << 3) + 4 * (m16 & 1);
        return o;
    }

    // ---- one (token, block) unit: S^T = K Q^T, online softmax, O^T += V^T P^T
    __device__ static inline void unit(TokState &st, const uint16_t *stage, const LaneOffs &lo, int lane, bool diag,
                                       int key_limit, float c) {
        const int g = lane >> 4;
        f32x4 acc[4];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            acc[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(stage + kt * 16 * D + lo.kx[s]);
                acc[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, st.qf[s], acc[kt], 0, 0, 0);
            }
        }
        // acc[kt][r] is key 16*kt + 4*g + r of the block, for head lane%16
        if (diag) {
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (16 * kt + 4 * g + r > key_limit) acc[kt][r] = -INFINITY;
        }
        float mx = acc[0][0];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r) mx = fmaxf(mx, acc[kt][r]);
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        if (__any(mx > st.m)) {          // some head's running max moved: rescale (rare after the first blocks)
            const float m_new = fmaxf(st.m, mx);
            const float alpha = fast_exp2((st.m - m_new) * c);
            st.m = m_new;
            st.l *= alpha;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) st.o[dt] *= alpha;
        }
        const float mc = st.m * c;
        float ls = 0.f;
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                acc[kt][r] = fast_exp2(acc[kt][r] * c - mc);
                ls += acc[kt][r];
            }
        st.l += ls;
        // P^T as B operand of k-step s2 (keys 32*s2 ..): slots 0-3 = keys 32*s2 + 4g + r, slots 4-7 = +16
        bf16x8 pb[2];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                pb[s2][r] = (__bf16)acc[2 * s2][r];
                pb[s2][4 + r] = (__bf16)acc[2 * s2 + 1][r];
            }
        const uint16_t *vt = stage + TILE_ELEMS;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const short4v v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) short4v *)(vt + (32 * s2) * D + lo.vx[dt]));
                const short4v v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) short4v *)(vt + (32 * s2 + 16) * D + lo.vx[dt]));
                const short8v v8 = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
                st.o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v8), pb[s2], st.o[dt], 0, 0, 0);
            }
    }

    __device__ static void run(const AttnArgs &a, int num_tiles) {
        extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
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
        if (ne > 0) issue_block_load(a, kb, vb, dense ? 0 : list_j[0], len, stages, w, lane);

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
        const LaneOffs lo = lane_offsets(lane);

        __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
        __syncthreads();
        for (int e = 0; e < ne; ++e) {
            const int j = dense ? e : list_j[e];
            const uint32_t mk = dense ? full : masks[j];
            if (e + 1 < ne)
                issue_block_load(a, kb, vb, dense ? e + 1 : list_j[e + 1], len, stages + ((e + 1) & 1) * STAGE_ELEMS, w, lane);
            const uint16_t *stage = stages + (e & 1) * STAGE_ELEMS;
            const bool diag = j == bt;
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const int ti = i * NW + w;
                if (mk & (1u << ti)) unit(st[i], stage, lo, lane, diag, t0 + ti - j * kBlock, c);
            }
            __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);     // the next block has landed in LDS
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
    if (lds > 160 * 1024 - 64) return INFLLMV2_ERR_UNSUPPORTED;      // sequences beyond ~3M tokens
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
    static const char *cfg = getenv("INFLLMV2_ATTN_CFG");      // experiment switch
    if (cfg && !strcmp(cfg, "8x2")) return launch_tile<8, 2>(L, a, cu_h);
    if (cfg && !strcmp(cfg, "8x4")) return launch_tile<8, 4>(L, a, cu_h);
    if (cfg && !strcmp(cfg, "16x2")) return launch_tile<16, 2>(L, a, cu_h);
    if (cfg && !strcmp(cfg, "4x4")) return launch_tile<4, 4>(L, a, cu_h);
    return launch_tile<16, 1>(L, a, cu_h);
}

}  // namespace ifv2
