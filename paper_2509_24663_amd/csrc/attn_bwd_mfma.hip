// Gradients of stage 4 on the matrix cores for the paper's head shape (bf16, 16 query heads per KV head,
// d_h = 128).  Same mathematics as attn_bwd.hip (chain rule on O = softmax(scale q K^T) V with the stored
// log-sum-exp; the paper prints no backward algorithm):
//     P = exp(z - lse),  dP = dO V^T,  dZ = P o (dP - Delta),  dQ = scale dZ K,  dK = scale dZ^T Q,  dV = P^T dO.
// Every product is an MFMA with the 16 heads of a token as one matrix dimension.  Operands go from global
// memory through LDS stages into MFMA registers.  Two small pre-passes write into stream-ordered scratch:
//   prep : Delta = <dO, O> and lse * log2(e) per (token, query head), token-major
//   kt   : per 64-key block K^T as [128 dims][64 keys]
//   dq   : one wavefront per (token, KV head), a workgroup of consecutive tokens walking the union of their
//          block lists with each block's K, V, K^T staged once in LDS.  Per 16 keys:
//          S^T = K Q^T and dP^T = V dO^T (4 + 4 MFMA 16x16x32: keys x heads), dZ^T in registers with one head per
//          lane, dQ^T += K^T dZ^T (8 MFMA 16x16x16: dims x heads).
//   dkv  : one workgroup of 4 wavefronts per (64-key block, chunk of later tokens, KV head); wavefront w owns keys
//          16 w .. 16 w + 15 with their K and V fragments in registers.  The workgroup lists the tokens of its
//          chunk that selected the block; per token S = Q K^T and dP = dO V^T (heads x keys), then
//          dV += P^T dO and dK += dZ^T Q (8 + 8 MFMA 16x16x16: keys x dims, contraction over the 16 heads; the
//          B operands, heads x dims, are read from the same row-major tiles with the transposing LDS read).
//          The four wavefronts share each token's Q and dO rows (8 KB) through a double-buffered LDS stage,
//          two tokens per barrier, the next two in flight in registers.  Results are added to the float32 outputs with
//          the L2's float atomics, one add per element and workgroup.
// Measured at 131072 tokens, 64 selected blocks: dq 31 ms, dkv 45 ms (the forward attention kernel: 12.6 ms; 3.5x
// its flops).  dkv is bound by the 8 KB of Q and dO rows it fetches per (token, block) -- tokens that selected a
// given block are scattered, so nothing is shared between blocks -- and dq by LDS traffic and barriers.
#include <algorithm>

#include <cstdlib>
#include "common.h"

namespace ifv2 {

namespace {

constexpr int D = 128, G = 16;
constexpr float LOG2E = 1.4426950408889634f;
constexpr int DKV_CHUNK = 2048;          // tokens per dkv workgroup

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef short short4v __attribute__((ext_vector_type(4)));

__device__ inline float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }
// four floats -> four bf16 (round to nearest even, the hardware conversion)
__device__ inline short4v to_bf16x4(float a, float b, float c, float d) {
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    const bf16x4 r = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};
    return __builtin_bit_cast(short4v, r);
}

struct BwdM {
    const uint16_t *q, *k, *v, *out, *dout;
    const float *lse;
    const int32_t *idx;          // nullptr: dense
    int topk_total, dense_below, hq;
    float scale;
    RowMap map;
    // scratch
    float *lse2, *delta;         // [T][hq]
    uint16_t *kt;                // [hkv][blocks][128][64]
    int64_t nblocks;             // 64-key blocks over all sequences
    uint32_t *sel_bits;          // [hkv][sel_words]: per sequence and key block, one bit per token that selected it
    int64_t sel_words;           //   (block-major, rows of ceil(len / 32) words); nullptr: not built (too large)
    // results
    uint16_t *dq;
    float *dk, *dv;
};

// first 64-key block of sequence seq in the packed block numbering
__device__ inline int block_base(const RowMap &m, int seq) {
    int b = 0;
    for (int s = 0; s < seq; ++s) b += (m.cu[s + 1] - m.cu[s] + kBlock - 1) / kBlock;
    return b;
}

// ------------------------------------------------------------------------------------------ pre-passes
__global__ void __launch_bounds__(256) bwd_prep_kernel(BwdM a) {
    // 16 threads per (token, query head): Delta = <dO, O>, and lse in the log2 domain, both token-major
    const int row = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
    const int head = tid >> 4, d0 = (tid & 15) * 8;
    const int64_t off = ((int64_t)row * a.hq + h * G + head) * D + d0;
    const uint4 rg = *reinterpret_cast<const uint4 *>(a.dout + off);
    const uint4 ro = *reinterpret_cast<const uint4 *>(a.out + off);
    const uint32_t wg[4] = {rg.x, rg.y, rg.z, rg.w}, wo[4] = {ro.x, ro.y, ro.z, ro.w};
    float dot = 0.f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        dot += __uint_as_float(wg[e] << 16) * __uint_as_float(wo[e] << 16);
        dot += __uint_as_float(wg[e] & 0xffff0000u) * __uint_as_float(wo[e] & 0xffff0000u);
    }
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) dot += __shfl_xor(dot, o);
    if ((tid & 15) == 0) {
        const int qh = h * G + head;
        a.delta[(int64_t)row * a.hq + qh] = dot;
        a.lse2[(int64_t)row * a.hq + qh] = a.lse[qhead_row(a.map, qh, a.hq, row)] * LOG2E;
    }
}

// words of the selection bitmap before sequence seq
__device__ inline int64_t sel_base(const RowMap &m, int seq) {
    int64_t w = 0;
    for (int s = 0; s < seq; ++s) {
        const int len = m.cu[s + 1] - m.cu[s];
        w += (int64_t)((len + kBlock - 1) / kBlock) * ((len + 31) / 32);
    }
    return w;
}

// Inverse of the block lists: bit t of row j says that token t selected key block j.  The dK/dV kernel then gets
// the tokens of a (block, 2048-token chunk) pair with one 256-byte read instead of searching every token's list.
// One workgroup per 256 tokens of a sequence; a wavefront reads a token's list with one coalesced load (lane =
// list entry) and takes its 64 tokens in turn.
__global__ void __launch_bounds__(256) bwd_sel_bits_kernel(BwdM a) {
    __shared__ int s_seq, s_tile;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, h = blockIdx.y;
    if (tid == 0) {
        int rem = blockIdx.x, s = 0;
        for (; s < a.map.batch; ++s) {
            const int nt = (a.map.cu[s + 1] - a.map.cu[s] + 255) / 256;
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
    if (len < a.dense_below) return;                  // dense sequences need no lists
    const int words = (len + 31) / 32;
    uint32_t *rows = a.sel_bits + (int64_t)h * a.sel_words + sel_base(a.map, seq);
    const int t_first = s_tile * 256 + w * 64, t_end = min(t_first + 64, len);
    for (int t = t_first; t < t_end; ++t) {
        const int bt = t / kBlock;
        const int32_t *e = a.idx + head_row(a.map, h, tok0 + t) * a.topk_total;
        for (int i = lane; i < a.topk_total; i += 64) {
            const int j = e[i];
            if (j >= 0 && j <= bt) atomicOr(rows + (int64_t)j * words + (t >> 5), 1u << (t & 31));
        }
    }
}

__global__ void __launch_bounds__(256) bwd_kt_kernel(BwdM a) {
    constexpr int KS = kBlock + 8;
    __shared__ __attribute__((aligned(16))) uint16_t tk[D][KS];
    __shared__ int s_seq, s_j;
    const int tid = threadIdx.x, h = blockIdx.y;
    if (tid == 0) {
        int rem = blockIdx.x, s = 0;
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
    const uint16_t *kb = a.k + (int64_t)tok0 * a.map.kv_tok_stride + (int64_t)h * a.map.kv_head_stride;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int c = tid + r * 256, key = c >> 4, d0 = (c & 15) * 8, u = j * kBlock + key;
        uint4 raw = make_uint4(0, 0, 0, 0);
        if (u < len) raw = *reinterpret_cast<const uint4 *>(kb + (int64_t)u * a.map.kv_tok_stride + d0);
        const uint32_t wd[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            tk[d0 + 2 * e][key] = (uint16_t)(wd[e] & 0xffffu);
            tk[d0 + 2 * e + 1][key] = (uint16_t)(wd[e] >> 16);
        }
    }
    __syncthreads();
    uint16_t *dst = a.kt + ((int64_t)h * a.nblocks + blockIdx.x) * (D * kBlock);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int c = tid + r * 256, d = c >> 3, k0 = (c & 7) * 8;
        *reinterpret_cast<uint4 *>(dst + d * kBlock + k0) = *reinterpret_cast<const uint4 *>(&tk[d][k0]);
    }
}

__global__ void __launch_bounds__(256) bwd_fill_zero_kernel(float4 *p, int64_t n4) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (int64_t)gridDim.x * 256)
        p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

// ------------------------------------------------------------------------------------------ dQ
// A workgroup owns NT consecutive tokens of one sequence and KV head, one wavefront per token.  Neighbouring
// tokens select mostly the same blocks, so the workgroup walks the union of their lists in ascending order and
// stages each block's K, V and K^T once in LDS for every wavefront whose token selected it (bitmaps in LDS say
// who did).  Two LDS stages: the next block is written to the other stage and the one after it is in flight in
// registers while the current one is computed.
constexpr int DQ_MAX_BLOCKS = 4096;      // blocks per sequence the bitmaps cover (262144 tokens)

template <int NT>
__global__ void __launch_bounds__(NT * 64) bwd_dq_mfma_kernel(BwdM a, int num_tiles) {
    constexpr int NTHR = NT * 64, CH = 1024 / NTHR;          // 16-byte chunks of a 16 KB tile per thread
    constexpr int KS = D + 8, TS = kBlock + 8;                // padded rows of the K / V tiles and of the K^T tile
    constexpr int STAGE = 2 * kBlock * KS + D * TS;           // K, V, K^T of one block
    extern __shared__ __attribute__((aligned(16))) uint16_t dq_smem[];      // two stages
    __shared__ uint32_t ubm[DQ_MAX_BLOCKS / 32], wbm[NT][DQ_MAX_BLOCKS / 32];
    __shared__ int s_seq, s_tile;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, h = blockIdx.y;
    if (tid == 0) {
        int rem = blockIdx.x, s = 0;
        for (; s < a.map.batch; ++s) {
            const int nt = (a.map.cu[s + 1] - a.map.cu[s] + NT - 1) / NT;
            if (rem < nt) break;
            rem -= nt;
        }
        s_seq = s;
        s_tile = rem;
    }
    for (int i = tid; i < DQ_MAX_BLOCKS / 32; i += NTHR) ubm[i] = 0;
    for (int i = tid; i < NT * (DQ_MAX_BLOCKS / 32); i += NTHR) (&wbm[0][0])[i] = 0;
    __syncthreads();
    const int seq = s_seq;
    if (seq >= a.map.batch) return;
    const int tok0 = a.map.cu[seq], len = a.map.cu[seq + 1] - tok0;
    const int t = s_tile * NT + w;                            // this wavefront's token
    const bool active = t < len;
    const int row = tok0 + min(t, len - 1), bt = min(t, len - 1) / kBlock;
    const bool dense = a.idx == nullptr || len < a.dense_below;
    // ---- who needs which block
    if (active) {
        if (dense) {
            for (int wd = lane; wd <= bt >> 5; wd += 64) {
                const uint32_t bits = wd < bt >> 5 ? 0xffffffffu : 0xffffffffu >> (31 - (bt & 31));
                wbm[w][wd] = bits;
                atomicOr(&ubm[wd], bits);
            }
        } else {
            const int32_t *my_idx = a.idx + head_row(a.map, h, row) * a.topk_total;
            for (int e = lane; e < a.topk_total; e += 64) {
                const int j = my_idx[e];
                if (j >= 0 && j <= bt) {
                    atomicOr(&wbm[w][j >> 5], 1u << (j & 31));
                    atomicOr(&ubm[j >> 5], 1u << (j & 31));
                }
            }
        }
    }
    __syncthreads();
    const int j_last = min(s_tile * NT + NT - 1, len - 1) / kBlock;    // last block any token of the tile can see
    auto next_needed = [&](int from) -> int {                        // first j >= from in the union, or -1
        for (int wd = from >> 5; wd <= j_last >> 5; ++wd) {
            uint32_t bits = ubm[wd];
            if (wd == from >> 5) bits &= 0xffffffffu << (from & 31);
            if (bits) return wd * 32 + __ffs(bits) - 1;
        }
        return -1;
    };

    const int n16 = lane & 15, g = lane >> 4;
    const int qh = h * G + n16;                                   // this lane's head
    bf16x8 qf[4], gf[4];                                          // Q and dO rows of head n16 as B operands
    {
        const uint16_t *qp = a.q + ((int64_t)row * a.hq + qh) * D + g * 8;
        const uint16_t *gp = a.dout + ((int64_t)row * a.hq + qh) * D + g * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            qf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(qp + ks * 32));
            gf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(gp + ks * 32));
        }
    }
    const float nlse2 = -a.lse2[(int64_t)row * a.hq + qh], delta = a.delta[(int64_t)row * a.hq + qh];
    const float c = a.scale * LOG2E;
    const uint16_t *kb = a.k + (int64_t)tok0 * a.map.kv_tok_stride + (int64_t)h * a.map.kv_head_stride;
    const uint16_t *vb = a.v + (int64_t)tok0 * a.map.kv_tok_stride + (int64_t)h * a.map.kv_head_stride;
    const uint16_t *ktb = a.kt + ((int64_t)h * a.nblocks + block_base(a.map, seq)) * (D * kBlock);
    f32x4 acc[8];                                                 // dQ^T: dims 16 dt + 4 g + r, head n16
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    struct BlkPre { uint4 k[CH], v[CH], kt[CH]; };
    auto gload = [&](int j) -> BlkPre {
        BlkPre pr;
#pragma unroll
        for (int r = 0; r < CH; ++r) {
            const int cc = tid + r * NTHR;
            const int64_t ro = (int64_t)min(j * kBlock + (cc >> 4), len - 1) * a.map.kv_tok_stride + (cc & 15) * 8;
            pr.k[r] = *reinterpret_cast<const uint4 *>(kb + ro);
            pr.v[r] = *reinterpret_cast<const uint4 *>(vb + ro);
            pr.kt[r] = reinterpret_cast<const uint4 *>(ktb + (int64_t)j * (D * kBlock))[cc];
        }
        return pr;
    };
    auto lstore = [&](const BlkPre &pr, int buf) {
        uint16_t *k_d = dq_smem + buf * STAGE, *v_d = k_d + kBlock * KS, *kt_d = v_d + kBlock * KS;
#pragma unroll
        for (int r = 0; r < CH; ++r) {
            const int cc = tid + r * NTHR;
            *reinterpret_cast<uint4 *>(k_d + (cc >> 4) * KS + (cc & 15) * 8) = pr.k[r];
            *reinterpret_cast<uint4 *>(v_d + (cc >> 4) * KS + (cc & 15) * 8) = pr.v[r];
            *reinterpret_cast<uint4 *>(kt_d + (cc >> 3) * TS + (cc & 7) * 8) = pr.kt[r];
        }
    };
    // Two LDS stages: while block j is consumed from one, block jn (already in registers) is written to the other
    // and block jnn is requested from memory; one barrier per block.
    int j = next_needed(0);
    int jn = j >= 0 ? next_needed(j + 1) : -1;
    int buf = 0;
    if (j >= 0) lstore(gload(j), 0);
    BlkPre cur = gload(jn >= 0 ? jn : max(j, 0));
    __syncthreads();
    while (j >= 0) {
        const uint16_t *k_s = dq_smem + buf * STAGE, *v_s = k_s + kBlock * KS, *kt_s = v_s + kBlock * KS;
        int jnn = -1;
        if (jn >= 0) {
            lstore(cur, buf ^ 1);                                    // its last readers passed the previous barrier
            jnn = next_needed(jn + 1);
            cur = gload(jnn >= 0 ? jnn : jn);                        // (past the last block: loaded again, unused)
        }
        const bool mine = active && ((wbm[w][j >> 5] >> (j & 31)) & 1u);
        if (mine) {
            const int key_limit = j == bt ? t - j * kBlock : kBlock;    // keys 0 .. limit of the block are visible
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) {
                if (16 * kt > key_limit) break;                          // wave-uniform
                f32x4 st = f32x4{0.f, 0.f, 0.f, 0.f}, dpt = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(k_s + (16 * kt + n16) * KS + g * 8 + ks * 32);
                    const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(v_s + (16 * kt + n16) * KS + g * 8 + ks * 32);
                    st = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[ks], st, 0, 0, 0);
                    dpt = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, gf[ks], dpt, 0, 0, 0);
                }
                float dz[4];                                             // element r: key 16 kt + 4 g + r, head n16
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float p = 16 * kt + 4 * g + r <= key_limit ? exp2_fast(__builtin_fmaf(st[r], c, nlse2)) : 0.f;
                    dz[r] = p * (dpt[r] - delta);
                }
                const short4v dzb = to_bf16x4(dz[0], dz[1], dz[2], dz[3]);
                // dQ^T (dims x heads) += K^T (dims x keys) dZ^T (keys x heads); A: row 16 dt + n16 of K^T, keys 16 kt + 4 g ..
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) {
                    const short4v ka = *reinterpret_cast<const short4v *>(kt_s + (16 * dt + n16) * TS + 16 * kt + 4 * g);
                    acc[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ka, dzb, acc[dt], 0, 0, 0);
                }
            }
        }
        __syncthreads();
        j = jn;
        jn = jnn;
        buf ^= 1;
    }
    if (!active) return;
    uint16_t *dq = a.dq + ((int64_t)row * a.hq + qh) * D + 4 * g;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
        uint2 pk;
        pk.x = (uint32_t)float_to_bf16(acc[dt][0] * a.scale) | ((uint32_t)float_to_bf16(acc[dt][1] * a.scale) << 16);
        pk.y = (uint32_t)float_to_bf16(acc[dt][2] * a.scale) | ((uint32_t)float_to_bf16(acc[dt][3] * a.scale) << 16);
        *reinterpret_cast<uint2 *>(dq + 16 * dt) = pk;
    }
}

// ------------------------------------------------------------------------------------------ dK, dV
// is block j in the ascending, -1 padded list e[0 .. n)?
__device__ inline bool list_has(const int32_t *e, int n, int j) {
    int lo = 0, hi = n;
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        const int x = e[mid];
        if (x >= 0 && x < j) lo = mid + 1; else hi = mid;
    }
    return lo < n && e[lo] == j;
}

constexpr int DKV_QS = D + 8;                                   // padded row of the row-major Q / dO tiles
constexpr int DKV_TOK_ELEMS = 2 * G * DKV_QS;                   // Q and dO rows of one token
constexpr int DKV_TB = 2;                                       // tokens per barrier (and per prefetch)

__global__ void __launch_bounds__(256) bwd_dkv_mfma_kernel(BwdM a) {
    constexpr int QS = DKV_QS, TOK_ELEMS = DKV_TOK_ELEMS, TB = DKV_TB;
    __shared__ __attribute__((aligned(16))) uint16_t tok_s[2 * TB * TOK_ELEMS];     // [2 buffers][TB tokens]
    __shared__ __attribute__((aligned(16))) float f_s[2][TB][32];  // lse * log2(e) and Delta of the 16 heads
    __shared__ int s_seq, s_j, s_list[DKV_CHUNK], s_wave_cnt[4];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int h = blockIdx.z;
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
    const int c0 = blockIdx.x * DKV_CHUNK, c1 = min(c0 + DKV_CHUNK, len);
    if (c1 <= j * kBlock || c0 >= len) return;
    const bool dense = a.idx == nullptr || len < a.dense_below;

    // ---- tokens of the chunk that selected the block, in token order
    int total = 0;
    if (!dense && a.sel_bits != nullptr) {
        // from the selection bitmap: the chunk is 64 words of the block's row; thread tid expands byte tid of them
        static_assert(DKV_CHUNK == 8 * 256, "one byte of the chunk's bits per thread");
        const int words = (len + 31) / 32;
        const uint32_t *row = a.sel_bits + (int64_t)h * a.sel_words + sel_base(a.map, seq) + (int64_t)j * words + (c0 >> 5);
        const int nw = (c1 - c0 + 31) >> 5;
        const uint32_t wv = (tid >> 2) < nw ? row[tid >> 2] : 0u;
        const uint32_t bits = (wv >> (8 * (tid & 3))) & 0xffu;
        const int cnt = __popc(bits);
        int incl = cnt;                                        // inclusive prefix inside the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o);
            if (lane >= o) incl += up;
        }
        if (lane == 63) s_wave_cnt[w] = incl;
        __syncthreads();
        int base = incl - cnt;
        for (int x = 0; x < 4; ++x) {
            if (x < w) base += s_wave_cnt[x];
            total += s_wave_cnt[x];
        }
        for (uint32_t rest = bits; rest; rest &= rest - 1) s_list[base++] = c0 + 8 * tid + __ffs(rest) - 1;
        __syncthreads();
    } else
    for (int r0 = c0; r0 < c1; r0 += 256) {
        const int t_mine = r0 + tid;
        bool sel = t_mine < c1 && t_mine >= j * kBlock;
        if (sel && !dense) sel = list_has(a.idx + head_row(a.map, h, tok0 + t_mine) * a.topk_total, a.topk_total, j);
        const uint64_t bal = __ballot(sel);
        if (lane == 0) s_wave_cnt[w] = __popcll(bal);
        __syncthreads();
        int base = total;
        for (int x = 0; x < 4; ++x) {
            if (x < w) base += s_wave_cnt[x];
            total += s_wave_cnt[x];
        }
        if (sel) s_list[base + __popcll(bal & ((1ull << lane) - 1ull))] = t_mine;
        __syncthreads();
    }
    if (total == 0) return;

    const int n16 = lane & 15, g = lane >> 4;
    // K and V rows of key 16 w + n16 as B operands (k = 8 dims at 32 ks + 8 g); rows past the sequence are never
    // visible to any token (causal), their contributions are masked to zero
    const int key = j * kBlock + 16 * w + n16;
    bf16x8 kf[4], vf[4];
    {
        const int64_t base = (int64_t)tok0 * a.map.kv_tok_stride + (int64_t)h * a.map.kv_head_stride +
                             (int64_t)min(key, len - 1) * a.map.kv_tok_stride + g * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            kf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(a.k + base + ks * 32));
            vf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(a.v + base + ks * 32));
        }
    }
    const float c = a.scale * LOG2E;
    f32x4 acc_k[8], acc_v[8];                  // rows: keys 16 w + 4 g + r; columns: dims 16 dt + n16
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
        acc_k[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        acc_v[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // The four wavefronts need the same per-token data, so it goes through LDS once: Q and dO rows (row-major,
    // padded: A operands), Q^T and dO^T ([dims][heads]: B operands), Delta and lse.  Double buffered, the next
    // token's 16 KB are in flight in registers while the current token is computed; one barrier per token.
    struct TokPre { uint4 q, g; float f; };
    auto gload = [&](int t) -> TokPre {
        TokPre pr;
        const int row = tok0 + t;
        const int64_t off = ((int64_t)row * a.hq + h * G + (tid >> 4)) * D + (tid & 15) * 8;
        pr.q = *reinterpret_cast<const uint4 *>(a.q + off);
        pr.g = *reinterpret_cast<const uint4 *>(a.dout + off);
        pr.f = (tid < 16 ? a.lse2 : a.delta)[(int64_t)row * a.hq + h * G + (tid & 15)];    // used by threads 0..31
        return pr;
    };
    auto lstore = [&](int buf, int slot, const TokPre &pr) {
        uint16_t *b = tok_s + (buf * TB + slot) * TOK_ELEMS;
        *reinterpret_cast<uint4 *>(b + (tid >> 4) * QS + (tid & 15) * 8) = pr.q;
        *reinterpret_cast<uint4 *>(b + G * QS + (tid >> 4) * QS + (tid & 15) * 8) = pr.g;
        if (tid < 32) f_s[buf][slot][tid] = pr.f;
    };
    // B operands of the two head-contractions come from the same row-major tiles through the transposing LDS
    // read: in each group of 16 lanes, lane L points at dims 4 (L % 4) .. + 3 of row L / 4 of a 4 x 16 block and
    // receives column L of it.  Block = heads 4 g .. 4 g + 3, dims 16 dt .. 16 dt + 15.
    typedef __attribute__((address_space(3))) short4v lds_s4;
    const int tr_off = (4 * g + (n16 >> 2)) * QS + 4 * (n16 & 3);
    // batches of TB tokens: batch i = list entries TB i .. TB i + TB - 1 (entries past the end repeat the last one
    // and are not computed)
    const int nbatch = (total + TB - 1) / TB;
    TokPre nxt[TB];
#pragma unroll
    for (int sl = 0; sl < TB; ++sl) lstore(0, sl, gload(s_list[min(sl, total - 1)]));
    __syncthreads();
    for (int ib = 0; ib < nbatch; ++ib) {
#pragma unroll
        for (int sl = 0; sl < TB; ++sl) nxt[sl] = gload(s_list[min((ib + 1) * TB + sl, total - 1)]);
#pragma unroll
        for (int sl = 0; sl < TB; ++sl) {
            const int it = ib * TB + sl;
            if (it >= total) break;                                  // uniform
            const int t = s_list[it];
            const uint16_t *b = tok_s + ((ib & 1) * TB + sl) * TOK_ELEMS;
            // A operands: Q and dO rows of head n16
            f32x4 sacc = f32x4{0.f, 0.f, 0.f, 0.f}, dpacc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const bf16x8 qa = *reinterpret_cast<const bf16x8 *>(b + n16 * QS + g * 8 + ks * 32);
                const bf16x8 ga = *reinterpret_cast<const bf16x8 *>(b + G * QS + n16 * QS + g * 8 + ks * 32);
                sacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa, kf[ks], sacc, 0, 0, 0);
                dpacc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ga, vf[ks], dpacc, 0, 0, 0);
            }
            // element r: head 4 g + r, key n16 of this wave's tile
            const float4 l2 = *reinterpret_cast<const float4 *>(&f_s[ib & 1][sl][4 * g]);
            const float4 dl = *reinterpret_cast<const float4 *>(&f_s[ib & 1][sl][16 + 4 * g]);
            const float l2a[4] = {l2.x, l2.y, l2.z, l2.w}, dla[4] = {dl.x, dl.y, dl.z, dl.w};
            const bool visible = key <= t;
            float p[4], dz[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                p[r] = visible ? exp2_fast(__builtin_fmaf(sacc[r], c, -l2a[r])) : 0.f;
                dz[r] = p[r] * (dpacc[r] - dla[r]);
            }
            const short4v pb = to_bf16x4(p[0], p[1], p[2], p[3]), dzb = to_bf16x4(dz[0], dz[1], dz[2], dz[3]);
            // dV (keys x dims) += P^T (keys x heads) dO (heads x dims); B: dim 16 dt + n16, heads 4 g .. 4 g + 3
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                const short4v qb = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4 *)(b + tr_off + 16 * dt));
                const short4v gb = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4 *)(b + G * QS + tr_off + 16 * dt));
                acc_v[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(pb, gb, acc_v[dt], 0, 0, 0);
                acc_k[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(dzb, qb, acc_k[dt], 0, 0, 0);
            }
        }
        if (ib + 1 < nbatch) {
#pragma unroll
            for (int sl = 0; sl < TB; ++sl) lstore((ib + 1) & 1, sl, nxt[sl]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int u = j * kBlock + 16 * w + 4 * g + r;
        if (u < len) {
            float *dk = a.dk + ((int64_t)h * a.map.total_rows + tok0 + u) * D + n16;
            float *dv = a.dv + ((int64_t)h * a.map.total_rows + tok0 + u) * D + n16;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                unsafeAtomicAdd(dk + 16 * dt, acc_k[dt][r] * a.scale);       // the L2's own float add, no CAS loop
                unsafeAtomicAdd(dv + 16 * dt, acc_v[dt][r]);
            }
        }
    }
}

}  // namespace

bool bwd_mfma_params(const infllmv2_params *p) {
    return p->dtype == INFLLMV2_BF16 && p->head_dim == D && p->num_q_heads / p->num_kv_heads == G;
}

// two [hq, rows] float arrays (lse in powers of two, <dO, O>), K^T tiles, and optionally the selection bitmap
size_t bwd_mfma_ws_bytes(const infllmv2_params *p, const BatchTotals &t, bool with_bitmap) {
    const size_t b_f = align256((size_t)t.rows * p->num_q_heads * sizeof(float));
    const size_t b_kt = align256((size_t)p->num_kv_heads * t.blocks * D * kBlock * sizeof(uint16_t));
    const size_t words = (size_t)(t.sel_words + 3) / 4 * 4;
    const size_t b_sel = with_bitmap ? align256((size_t)p->num_kv_heads * words * sizeof(uint32_t)) : 0;
    return 2 * b_f + b_kt + b_sel;
}

// Returns INFLLMV2_ERR_UNSUPPORTED (nothing launched) for shapes this path does not cover.
int launch_attn_bwd_mfma(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx,
                         int dense_below, const void *out, const float *lse, const void *dout, void *dq, float *dk,
                         float *dv, const int32_t *cu_h) {
    const infllmv2_params *p = L.p;
    if (!bwd_mfma_params(p)) return INFLLMV2_ERR_UNSUPPORTED;
    if ((((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out | (uintptr_t)dout | (uintptr_t)dq) & 15) != 0 ||
        L.map.kv_tok_stride % 8 != 0 || L.map.kv_head_stride % 8 != 0)
        return INFLLMV2_ERR_UNSUPPORTED;
    const int64_t rows = L.map.total_rows;
    if (rows == 0) return INFLLMV2_OK;
    int64_t nblocks = 0;
    for (int s = 0; s < L.map.batch; ++s) nblocks += (cu_h[s + 1] - cu_h[s] + kBlock - 1) / kBlock;
    const int hkv = p->num_kv_heads, hq = p->num_q_heads;
    if (nblocks > 65535 || hkv > 65535 || rows > 0x7fffffff / 4) return INFLLMV2_ERR_UNSUPPORTED;
    if ((L.max_len + kBlock - 1) / kBlock > DQ_MAX_BLOCKS) return INFLLMV2_ERR_UNSUPPORTED;
    const size_t b_f = align256((size_t)rows * hq * sizeof(float));
    const size_t b_kt = align256((size_t)hkv * nblocks * D * kBlock * sizeof(uint16_t));
    // selection bitmap (block-major): only when block lists exist and it stays moderate (it grows with len^2 / 2048
    // bytes per sequence and KV head: 32 MB at 128K tokens); otherwise the dK/dV kernel searches the lists
    int64_t sel_words = 0, sel_tiles = 0;
    if (idx != nullptr)
        for (int s = 0; s < L.map.batch; ++s) {
            const int64_t len = cu_h[s + 1] - cu_h[s];
            sel_words += ((len + kBlock - 1) / kBlock) * ((len + 31) / 32);
            sel_tiles += (len + 255) / 256;
        }
    sel_words = (sel_words + 3) / 4 * 4;                        // zeroed 16 bytes at a time
    // the bitmap is built when the caller's workspace has room for it
    const size_t b_sel_full = align256((size_t)hkv * sel_words * sizeof(uint32_t));
    char *ws = (char *)L.ws;
    if (ws == nullptr || L.ws_bytes < 2 * b_f + b_kt) return INFLLMV2_ERR_WORKSPACE_TOO_SMALL;
    const bool use_bits = idx != nullptr && sel_words > 0 && L.ws_bytes >= 2 * b_f + b_kt + b_sel_full;
    BwdM a;
    a.q = (const uint16_t *)q;
    a.k = (const uint16_t *)k;
    a.v = (const uint16_t *)v;
    a.out = (const uint16_t *)out;
    a.dout = (const uint16_t *)dout;
    a.lse = lse;
    a.idx = idx;
    a.topk_total = p->topk_total;
    a.dense_below = dense_below;
    a.hq = hq;
    a.scale = p->softmax_scale;
    a.map = L.map;
    a.lse2 = (float *)ws;
    a.delta = (float *)(ws + b_f);
    a.kt = (uint16_t *)(ws + 2 * b_f);
    a.nblocks = nblocks;
    a.sel_bits = use_bits ? (uint32_t *)(ws + 2 * b_f + b_kt) : nullptr;
    a.sel_words = sel_words;
    a.dq = (uint16_t *)dq;
    a.dk = dk;
    a.dv = dv;
    const int64_t n4 = rows * hkv * D / 4;
    const unsigned zg = (unsigned)std::min<int64_t>((n4 + 255) / 256, 8192);
    hipLaunchKernelGGL(bwd_fill_zero_kernel, dim3(zg), dim3(256), 0, L.stream, (float4 *)dk, n4);
    hipLaunchKernelGGL(bwd_fill_zero_kernel, dim3(zg), dim3(256), 0, L.stream, (float4 *)dv, n4);
    if (use_bits) {
        const int64_t s4 = (int64_t)hkv * sel_words / 4;
        hipLaunchKernelGGL(bwd_fill_zero_kernel, dim3((unsigned)std::min<int64_t>((s4 + 255) / 256, 8192)), dim3(256), 0,
                           L.stream, (float4 *)a.sel_bits, s4);
        hipLaunchKernelGGL(bwd_sel_bits_kernel, dim3((unsigned)sel_tiles, hkv), dim3(256), 0, L.stream, a);
    }
    hipLaunchKernelGGL(bwd_prep_kernel, dim3((unsigned)rows, hkv), dim3(256), 0, L.stream, a);
    hipLaunchKernelGGL(bwd_kt_kernel, dim3((unsigned)nblocks, hkv), dim3(256), 0, L.stream, a);
    constexpr int DQ_NT = 16;
    int64_t dq_tiles = 0;
    for (int s = 0; s < L.map.batch; ++s) dq_tiles += (cu_h[s + 1] - cu_h[s] + DQ_NT - 1) / DQ_NT;
    constexpr size_t dq_lds = 2 * (size_t)(2 * kBlock * (D + 8) + D * (kBlock + 8)) * sizeof(uint16_t);     // two stages
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(bwd_dq_mfma_kernel<DQ_NT>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)dq_lds) != hipSuccess)
        return INFLLMV2_ERR_HIP;
    hipLaunchKernelGGL(bwd_dq_mfma_kernel<DQ_NT>, dim3((unsigned)dq_tiles, hkv), dim3(DQ_NT * 64), dq_lds, L.stream, a,
                       (int)dq_tiles);
    const unsigned chunks = (unsigned)((L.max_len + DKV_CHUNK - 1) / DKV_CHUNK);
    hipLaunchKernelGGL(bwd_dkv_mfma_kernel, dim3(chunks, (unsigned)nblocks, hkv), dim3(256), 0, L.stream, a);
    return hip_status(hipGetLastError());
}

}  // namespace ifv2
