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

#include "attn_unit.h"

namespace ifv2 {

namespace {

using namespace attn_unit;

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

#ifdef IFV2_RING_PROF
__device__ unsigned long long g_prof[8];
#define PROF_DECL() long long prof_acc[5] = {0, 0, 0, 0, 0}
#define PROF_T0() const long long prof_t0 = __builtin_amdgcn_s_memtime()
#define PROF_ADD(slot) prof_acc[slot] += __builtin_amdgcn_s_memtime() - prof_t0
#define PROF_FLUSH() do { if (lane == 0) for (int i_ = 0; i_ < 5; ++i_) atomicAdd(&g_prof[i_], (unsigned long long)prof_acc[i_]); } while (0)
#else
#define PROF_DECL() do {} while (0)
#define PROF_T0() do {} while (0)
#define PROF_ADD(slot) do {} while (0)
#define PROF_FLUSH() do {} while (0)
#endif

template <int NW, int TPW, int S>
struct TileKernel {
    static constexpr int T = NW * TPW;
    static constexpr int NTHR = NW * 64;
    static constexpr bool RING = S > 2;       // S == 2: lock-step double buffering; S > 2: flag-driven ring
    static_assert(!RING || TPW == 1, "the ring schedule counts one consumer per wave");
    static_assert(32 % NW == 0 || NW == 32, "32 one-KB load instructions are dealt round-robin to the waves");

    // ---- block j of the sequence: global -> LDS stage (K tile then V tile), asynchronously; the 32 one-KB
    // pieces are dealt round-robin to the waves.
    __device__ static inline void issue_block_load(const AttnArgs &a, const uint16_t *kb, const uint16_t *vb, int j,
                                                   int len, uint16_t *stage, int w, int lane) {
#pragma unroll
        for (int qi = w; qi < 32; qi += NW)
            load_piece(qi < 16 ? kb : vb, a.map.kv_tok_stride, j, len, stage + (qi < 16 ? 0 : TILE_ELEMS), qi & 15, lane);
    }

    // ---- the same load issued by a single wave (ring schedule: the wave on duty for this entry)
    __device__ static inline void issue_block_load_wave(const AttnArgs &a, const uint16_t *kb, const uint16_t *vb, int j,
                                                        int len, uint16_t *stage, int lane) {
#pragma unroll 4
        for (int qi = 0; qi < 32; ++qi)
            load_piece(qi < 16 ? kb : vb, a.map.kv_tok_stride, j, len, stage + (qi < 16 ? 0 : TILE_ELEMS), qi & 15, lane);
    }

    // Per-entry state word of the ring schedule: bits 16.. count the load pieces that have landed (NW = all of
    // them), bits 0..15 count the waves that have finished consuming the entry.  Both only grow.
    __device__ static inline int st_ready(int v) { return v >> 16; }
    __device__ static inline int st_done(int v) { return v & 0xffff; }

    // Bounded waits on a state word.  They return false (and raise *err for the whole workgroup) if the bound
    // is hit, so that a logic error can never hang the GPU: every wave then leaves its loop.
    template <bool READY>
    __device__ static inline bool wait_state(volatile int *word, int target, volatile int *err) {
        int spins = 0;
        while ((READY ? st_ready(*word) : st_done(*word)) < target) {
            __builtin_amdgcn_s_sleep(1);
            if (++spins > (1 << 22) || *err) {
                *err = 1;
                return false;
            }
        }
        return true;
    }

    __device__ static void run(const AttnArgs &a, int num_tiles) {
        extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
        uint16_t *stages = smem;
        uint32_t *masks = reinterpret_cast<uint32_t *>(smem + S * STAGE_ELEMS);
        int32_t *list_j = reinterpret_cast<int32_t *>(masks + a.nb_cap);
        int *state = reinterpret_cast<int *>(list_j + a.list_cap);      // ring schedule: one word per union entry
        __shared__ int s_seq, s_tile, s_ne;

        const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
        const int h = blockIdx.y;
        // Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2).  Neighbouring tiles share most
        // of their K/V blocks, so runs of XG consecutive tiles are sent to the same XCD; late (long-context)
        // tiles go first.
        int lin = (int)blockIdx.x;
        {
            constexpr int XG = 4;
            const int full = num_tiles / (8 * XG) * (8 * XG);
            if (lin < full) {
                const int grp = lin / (8 * XG), r = lin % (8 * XG);
                lin = grp * (8 * XG) + (r % 8) * XG + r / 8;
            }
        }
        const int tile_id = num_tiles - 1 - lin;
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
        constexpr int PRE = RING ? S - 1 : 1;          // entries loaded cooperatively before the main loop
        for (int e = 0; e < PRE && e < ne; ++e)
            issue_block_load(a, kb, vb, dense ? e : list_j[e], len, stages + e * STAGE_ELEMS, w, lane);

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

        __shared__ int ring_err;
        if (RING) {
            for (int e = tid; e < ne; e += NTHR) state[e] = e < PRE ? NW << 16 : 0;     // preloaded entries are ready
            if (tid == 0) ring_err = 0;
        }
        __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
        __syncthreads();
        if (!RING) {
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
        } else {
            // Ring schedule.  Every wave walks the union list on its own and works only on the entries its token
            // selected, so waves are not held in lock step by the blocks they skip and their MFMA and VALU phases
            // drift apart and overlap.  Entry y = x + S - 1 is loaded while entry x is being consumed: by the first
            // wave that has no work at x (it would be idle anyway), or, when every wave is busy at x, by all of
            // them, two pieces each.  A loader first waits until every consumer of the stage's previous occupant
            // (entry x - 1) has finished, and publishes its pieces in the entry's state word once they have
            // landed.  Every wait is for an entry with a smaller number than anything the waiter still has to
            // publish, so waits cannot form a cycle; each wait is bounded anyway.
            volatile int *vstate = state, *err = &ring_err;
            constexpr uint32_t ALLW = NW >= 32 ? 0xffffffffu : ((1u << NW) - 1u);
            int pending = -1, pending_add = 0;
            bool ok = true;
            PROF_DECL();
            auto flush = [&]() {
                if (pending >= 0) {
                    PROF_T0();
                    __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
                    PROF_ADD(0);
                    if (lane == 0) atomicAdd(state + pending, pending_add << 16);
                    pending = -1;
                }
            };
            PROF_T0();
            for (int x = 0; x < ne && ok; ++x) {
                flush();                                 // a load issued while idle gets one entry of slack
                const int j = dense ? x : list_j[x];
                const uint32_t mk = dense ? full : masks[j];
                const bool mine = (mk >> w) & 1u;
                const int y = x + S - 1;
                if (y < ne) {
                    const uint32_t idle = ~mk & ALLW;
                    const bool solo = idle != 0u;
                    // loader = the (x mod #idle)-th idle wave, so that successive loads are issued by different
                    // waves and their latencies overlap
                    bool loader = true;
                    if (solo) {
                        const int pick = x % __popc(idle);
                        loader = ((idle >> w) & 1u) && __popc(idle & ((1u << w) - 1u)) == pick;
                    }
                    if (loader) {
                        flush();
                        if (x >= 1) {
                            const int jp = dense ? x - 1 : list_j[x - 1];
                            PROF_T0();
                            ok = wait_state<false>(vstate + x - 1, __popc(dense ? full : masks[jp]), err);
                            PROF_ADD(1);
                        }
                        if (ok) {
                            uint16_t *dst = stages + (y % S) * STAGE_ELEMS;
                            const int jy = dense ? y : list_j[y];
                            if (solo) issue_block_load_wave(a, kb, vb, jy, len, dst, lane);
                            else issue_block_load(a, kb, vb, jy, len, dst, w, lane);
                            pending = y;
                            pending_add = solo ? NW : 1;
                        }
                    }
                }
                if (ok && mine) {
                    if (st_ready(vstate[x]) < NW) {
                        flush();
                        PROF_T0();
                        ok = wait_state<true>(vstate + x, NW, err);
                        PROF_ADD(2);
                    }
                    if (ok) {
                        // LDS-only ordering (no wait on this wave's own loads in flight): the tile reads below must
                        // not start before the state word was seen, and must be complete before the wave signs off
                        __builtin_amdgcn_s_waitcnt(WAIT_LGKMCNT0);
                        asm volatile("" ::: "memory");
                        PROF_T0();
                        unit(st[0], stages + (x % S) * STAGE_ELEMS, lo, lane, j == bt, t0 + w - j * kBlock, c);
                        asm volatile("" ::: "memory");
                        __builtin_amdgcn_s_waitcnt(WAIT_LGKMCNT0);
                        PROF_ADD(3);
                        if (lane == 0) atomicAdd(state + x, 1);
                        flush();
                    }
                }
            }
            flush();
            PROF_ADD(4);
            PROF_FLUSH();
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

template <int NW, int TPW, int S>
__global__ void __launch_bounds__(NW * 64) attn_tile_kernel(AttnArgs a, int num_tiles) {
    TileKernel<NW, TPW, S>::run(a, num_tiles);
}

template <int NW, int TPW, int S>
int launch_tile(const Launch &L, const AttnArgs &a0, const int32_t *cu_h) {
    constexpr int T = NW * TPW;
    AttnArgs a = a0;
    int64_t tiles = 0;
    for (int s = 0; s < L.map.batch; ++s) tiles += (cu_h[s + 1] - cu_h[s] + T - 1) / T;
    if (tiles == 0) return INFLLMV2_OK;
    const int nb_max = (L.max_len + kBlock - 1) / kBlock;
    a.nb_cap = a.idx ? (nb_max + 3) / 4 * 4 : 0;
    a.list_cap = a.idx ? min(nb_max, T * L.p->topk_total) : 0;
    const int state_cap = S > 2 ? nb_max : 0;                            // ring: one word per union entry
    const size_t lds = (size_t)S * STAGE_ELEMS * sizeof(uint16_t) + (size_t)(a.nb_cap + a.list_cap + state_cap) * 4;
    if (lds > 160 * 1024 - 256) return INFLLMV2_ERR_UNSUPPORTED;     // does not fit: the caller tries fewer stages
    auto kern = attn_tile_kernel<NW, TPW, S>;
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
    if (cfg && !strcmp(cfg, "8x2")) return launch_tile<8, 2, 2>(L, a, cu_h);
    if (cfg && !strcmp(cfg, "lock")) return launch_tile<16, 1, 2>(L, a, cu_h);
    if (cfg && !strcmp(cfg, "ring3")) return launch_tile<16, 1, 3>(L, a, cu_h);
    if (cfg && !strcmp(cfg, "ring4")) return launch_tile<16, 1, 4>(L, a, cu_h);
    return launch_tile<16, 1, 2>(L, a, cu_h);
}

#ifdef IFV2_RING_PROF
extern "C" void infllmv2_debug_prof(unsigned long long *out, int reset) {
    unsigned long long z[8] = {0};
    (void)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_prof), sizeof(z));
    if (reset) (void)hipMemcpyToSymbol(HIP_SYMBOL(g_prof), z, sizeof(z));
}
#endif

}  // namespace ifv2
