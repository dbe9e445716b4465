// Stage 2: S^shared = sum over the GQA group of softmax(scale * Q K^{C1 T})  (Sec. 3.3 Eq. 4-5).
// Both kernels follow the two-pass scheme of Alg. 1 / Sec. 3.4: pass 1 finds the log-sum-exp of
// every (token, head) row on chip, pass 2 recomputes the logits, normalises, sums the G heads of
// the group on chip and stores only the group sum.  Per-head score rows never reach HBM.
//
// LSE Approximation (Sec. 3.4, Eq. 7; lse_mode 1): pass 1 runs over the four times coarser keys K^{C2}
// instead.  K^{C2}_i is the mean of 4 l_C1 keys starting at 4 s_C1 i, i.e. (when s_C1 divides l_C1) the mean of
// the four disjoint K^{C1} windows 4i + m l_C1 / s_C1, m = 0..3, so it is formed on the fly from K^{C1} and
// needs no input of its own.  A row that sees no coarse key gets all-zero scores.

#include <type_traits>

#include "common.h"

namespace ifv2 {

// ------------------------------------------------------------------------------------------
// Generic fp32-arithmetic kernel: one workgroup per (query row, KV head); any G <= 16, d in {64,128},
// fp32 or bf16 inputs.  Used for fp32 data, unusual head shapes and single-row (decode) calls.
// ------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ void __launch_bounds__(256)
block_scores_generic(const T *__restrict__ q, const float *__restrict__ kc, RowMap map, int hq, int lc, int sc,
                     float scale, int dense_below, int lse_mode, float *__restrict__ s_shared, int64_t row_stride,
                     PoolArgs pool) {
    const int row = blockIdx.x, h = blockIdx.y;
    const int G = hq / map.num_kv_heads;
    const RowLoc loc = locate(map, row);
    const int v = visible_cmp(loc.pos, lc, sc);
    if (v == 0 || loc.len < dense_below) return;      // dense sequences need no scores
    // pass 1 runs over v1 keys: the fine ones, or the coarse ones made of `cstep`-spaced groups of four
    const int cstep = lc / sc;
    const int v1 = lse_mode == 0 ? v : min(visible_cmp(loc.pos, 4 * lc, 4 * sc), num_cmp(loc.len, 4 * lc, 4 * sc));
    if (v1 == 0) {                                    // no coarse key visible yet: all-zero scores
        float *out0 = s_shared + head_row(map, h, row) * row_stride;
        if (pool.on) {
            for (int j = threadIdx.x; j <= loc.pos / kBlock && max(pool.stride * j - pool.pad, 0) < v; j += 256) out0[j] = 0.f;
        } else {
            for (int i = threadIdx.x; i < v; i += 256) out0[i] = 0.f;
        }
        return;
    }
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
    for (int i = tid; i < v1; i += 256) {
        float z[kMaxGroup];
#pragma unroll
        for (int g = 0; g < kMaxGroup; ++g) z[g] = 0.f;
        const float *kr = kcb + (int64_t)(lse_mode == 0 ? i : 4 * i) * D;
        for (int c = 0; c < D; c += 4) {
            float4 kv = *reinterpret_cast<const float4 *>(kr + c);
            if (lse_mode != 0) {
                const float4 k1 = *reinterpret_cast<const float4 *>(kr + (int64_t)cstep * D + c);
                const float4 k2 = *reinterpret_cast<const float4 *>(kr + (int64_t)2 * cstep * D + c);
                const float4 k3 = *reinterpret_cast<const float4 *>(kr + (int64_t)3 * cstep * D + c);
                kv.x = ((kv.x + k1.x) + (k2.x + k3.x)) * 0.25f;
                kv.y = ((kv.y + k1.y) + (k2.y + k3.y)) * 0.25f;
                kv.z = ((kv.z + k1.z) + (k2.z + k3.z)) * 0.25f;
                kv.w = ((kv.w + k1.w) + (k2.w + k3.w)) * 0.25f;
            }
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
    auto score = [&](int i) -> float {
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
        return s;
    };
    if (pool.on) {
        // one thread per selection block up to the query's own: the max over its pooling window (Eq. 6), clipped
        // to the visible keys
        for (int j = tid; j <= loc.pos / kBlock && max(pool.stride * j - pool.pad, 0) < v; j += 256) {
            const int lo = pool.stride * j - pool.pad;
            float m = 0.f;
            for (int u = 0; u < pool.len; ++u)
                if (lo + u >= 0 && lo + u < v) m = fmaxf(m, score(lo + u));
            out[j] = m;
        }
    } else {
        for (int i = tid; i < v; i += 256) out[i] = score(i);
    }
}

template <typename T, int D>
static int launch_generic(const Launch &L, const void *q, const float *kc, float *s_shared, int64_t row_stride,
                          const PoolArgs &pool) {
    dim3 grid(L.map.total_rows, L.p->num_kv_heads);
    if (grid.x == 0) return INFLLMV2_OK;
    hipLaunchKernelGGL((block_scores_generic<T, D>), grid, dim3(256), 0, L.stream, (const T *)q, kc, L.map,
                       L.p->num_q_heads, L.p->cmp_len, L.p->cmp_stride, L.p->softmax_scale, L.p->dense_threshold,
                       L.p->lse_mode, s_shared, row_stride, pool);
    return hip_status(hipGetLastError());
}


// ------------------------------------------------------------------------------------------
// MFMA kernel for bf16 Q, G = 16, d = 128 (the paper's head shape).
//
// A workgroup owns T consecutive tokens of one KV head; every wave keeps the Q rows of its TPW tokens in
// registers as MFMA A operands (M = the 16 heads of the group).  Compressed keys stream through LDS in
// tiles of 64 and each B fragment read from LDS is reused by all TPW tokens of the wave.  A lane then owns
// one key column and four heads, so
//   pass 1 keeps a private running (reference, sum 2^(y - reference)) per head with no cross-lane traffic
//          in the loop; the reference is only moved when a logit exceeds it by 2^16, and
//   pass 2 sums its four heads in registers and finishes the head-group sum with a 3-step butterfly
//          across the four lane groups, after which the 64 lanes hold 64 consecutive keys' group sums.
//
// Precision.  The ranking of blocks is sensitive to ~1e-3 relative changes of the scores, so the operands
// are not rounded to bf16.  Q (bf16) converts to fp16 exactly and K^{C1} (float32 means of 32 keys) is
// rounded to fp16, whose 11-bit significand keeps the logit error near 1e-4 -- one fp16 MFMA instead of a
// bf16 high/low pair.  fp16's narrow exponent range is handled by exact power-of-two scalings: a token whose Q
// magnitudes would leave the range gets its own exponent, and a key tile that holds a magnitude above 2^15
// (never the case for real activations) is re-staged with its own shift; both are undone by a multiply on the
// accumulator, on a slower path.  Both passes see the same logits.
//
// Vector-instruction budget.  MFMA and vector instructions share one issue port, and a (token, key tile) pair
// has 16 MFMAs against 16 exponentials plus their sums, so every other vector instruction per logit shows up
// in the run time.  Two are avoided: softmax_scale * log2(e) is multiplied into K^{C1} when a tile is converted
// to fp16 (the conversion rounds anyway, so this adds no error), and the accumulator is seeded with minus the
// row's reference (pass 1) or minus its log-sum-exp (pass 2), so the MFMA result is the exponent itself.  The
// rare tiles or tokens that carry a power-of-two rescaling take a slower path with an explicit multiply.
// ------------------------------------------------------------------------------------------
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

namespace {

constexpr int SD = 128, SG = 16;
constexpr int SKS = SD + 8;                    // LDS row stride (fp16) of a compressed-key tile
constexpr int S_TILE = kBlock * SKS;           // one 64-key tile
constexpr float S_LOG2E = 1.4426950408889634f;
constexpr float S_SLACK = 16.0f;               // pass 1 moves its reference when a logit exceeds it by 2^16
constexpr float S_FP16_SAFE = 32768.0f;

// fp16 copy of the compressed keys in tiles of 64 rows (written by kc_half_kernel): per KV head `tiles` tiles of
// 64 x 128 halves, sequences back to back (sequence s starts at tile sum_{s' < s} ceil(nc(s') / 64)), rows past a
// sequence's last key are zero; tile values are K * cm * 2^-shift with the tile's shift stored beside.
struct HalfTiles {
    const _Float16 *data;
    const int32_t *shift;
    int32_t tiles;            // per KV head
};

struct ScoreArgs {
    const uint16_t *q;
    const float *kc;
    HalfTiles fine, coarse;   // K^{C1}; K^{C2} (only with the LSE Approximation)
    float *out;
    RowMap map;
    int hq, lc, sc, dense_below, lse_mode;
    float scale;
    int64_t row_stride;
};

__device__ inline float s_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// data-parallel-primitive moves of a 32-bit value: lane i receives the value of another lane without touching LDS
template <int CTRL>
__device__ inline unsigned dpp_move(unsigned x) {
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, true);
}
// max (MAX) or sum over the 16 lanes of a row (lanes with equal lane / 16), result in every lane: swaps inside quads,
// then the mirror images inside 8 and 16 lanes
template <bool MAX>
__device__ inline float row16_all(float x) {
    auto step = [](float v, float o) { return MAX ? fmaxf(v, o) : v + o; };
    x = step(x, __uint_as_float(dpp_move<0xB1>(__float_as_uint(x))));       // quad_perm [1,0,3,2]
    x = step(x, __uint_as_float(dpp_move<0x4E>(__float_as_uint(x))));       // quad_perm [2,3,0,1]
    x = step(x, __uint_as_float(dpp_move<0x141>(__float_as_uint(x))));      // row_half_mirror
    return step(x, __uint_as_float(dpp_move<0x140>(__float_as_uint(x))));   // row_mirror
}
constexpr int DPP_QUAD_SWAP1 = 0xB1;   // quad_perm [1,0,3,2]
constexpr int DPP_QUAD_SWAP2 = 0x4E;   // quad_perm [2,3,0,1]
constexpr int DPP_WAVE_SHR1 = 0x138;   // lane i <- lane i - 1 (lane 0 <- 0)

// Pre-pass of the matrix-core kernel: one workgroup per 64-row key tile.  Converts K^{C1} (or, for tiles
// >= fine.tiles, the coarse keys of Eq. 7: row i = mean of K^{C1} rows 4i + m l_C1/s_C1, m = 0..3) to fp16,
// multiplied by cm = the mantissa of softmax_scale * log2(e), and by 2^-shift where shift is the smallest power of
// two that brings the tile's largest magnitude below 2^15 (0 for any real activations).
__global__ void __launch_bounds__(256)
kc_half_kernel(const float *__restrict__ kc, RowMap map, int lc, int sc, int dense_below, float cm,
               _Float16 *__restrict__ fine, int32_t *__restrict__ sh_fine, int tiles_fine,
               _Float16 *__restrict__ coarse, int32_t *__restrict__ sh_coarse, int tiles_coarse) {
    __shared__ int s_seq, s_local;
    __shared__ float s_red[4];
    const int tid = threadIdx.x, h = blockIdx.y;
    const bool is_coarse = (int)blockIdx.x >= tiles_fine;
    const int tile = is_coarse ? blockIdx.x - tiles_fine : blockIdx.x;
    const int wl = is_coarse ? 4 * lc : lc, ws = is_coarse ? 4 * sc : sc;
    if (tid == 0) {
        int rem = tile, s = 0;
        for (; s < map.batch; ++s) {
            const int nt = (num_cmp(map.cu[s + 1] - map.cu[s], wl, ws) + kBlock - 1) / kBlock;
            if (rem < nt) break;
            rem -= nt;
        }
        s_seq = s;
        s_local = rem;
    }
    __syncthreads();
    const int seq = s_seq;
    if (seq >= map.batch) return;
    const int len = map.cu[seq + 1] - map.cu[seq];
    if (len < dense_below) return;                    // dense sequences are never scored
    const int rows = num_cmp(len, wl, ws), cstep = lc / sc;
    const float *kcb = kc + ((int64_t)h * map.kc_total_c + map.cu_c[seq]) * SD;
    float4 x[8];
    float amax = 0.f;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int c = tid + r * 256;
        const int row = s_local * kBlock + (c >> 5), col = (c & 31) * 4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row < rows) {
            if (!is_coarse) {
                v = *reinterpret_cast<const float4 *>(kcb + (int64_t)row * SD + col);
            } else {
                const float *b = kcb + (int64_t)4 * row * SD + col;
                const float4 k0 = *reinterpret_cast<const float4 *>(b);
                const float4 k1 = *reinterpret_cast<const float4 *>(b + (int64_t)cstep * SD);
                const float4 k2 = *reinterpret_cast<const float4 *>(b + (int64_t)2 * cstep * SD);
                const float4 k3 = *reinterpret_cast<const float4 *>(b + (int64_t)3 * cstep * SD);
                v.x = ((k0.x + k1.x) + (k2.x + k3.x)) * 0.25f;
                v.y = ((k0.y + k1.y) + (k2.y + k3.y)) * 0.25f;
                v.z = ((k0.z + k1.z) + (k2.z + k3.z)) * 0.25f;
                v.w = ((k0.w + k1.w) + (k2.w + k3.w)) * 0.25f;
            }
        }
        x[r] = v;
        amax = fmaxf(fmaxf(amax, fmaxf(fabsf(v.x), fabsf(v.y))), fmaxf(fabsf(v.z), fabsf(v.w)));
    }
    amax = wave_max(amax);
    if ((tid & 63) == 0) s_red[tid >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    if (!(amax < 3.0e38f)) amax = 3.0e38f;            // Inf / NaN inputs: keep going, results are Inf / NaN anyway
    int ek = 0;
    if (amax > 0.f) (void)frexpf(amax, &ek);          // amax < 2^ek and cm < 1
    const int shift = max(0, ek - 15);
    const float f = __builtin_ldexpf(cm, -shift);
    _Float16 *dst = (is_coarse ? coarse + ((int64_t)h * tiles_coarse + tile) * (kBlock * SD)
                               : fine + ((int64_t)h * tiles_fine + tile) * (kBlock * SD));
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int c = tid + r * 256;
        typedef _Float16 half4 __attribute__((ext_vector_type(4)));
        const half4 hv = {(_Float16)(x[r].x * f), (_Float16)(x[r].y * f), (_Float16)(x[r].z * f), (_Float16)(x[r].w * f)};
        *reinterpret_cast<half4 *>(dst + (c >> 5) * SD + (c & 31) * 4) = hv;
    }
    if (tid == 0) (is_coarse ? sh_coarse : sh_fine)[(int64_t)h * (is_coarse ? tiles_coarse : tiles_fine) + tile] = shift;
}

// W = 32: lanes 0..31 get x[lane] + x[lane + 32], lanes 32..63 get y[lane - 32] + y[lane].
// W = 16 (rows of 16 lanes): rows 0 and 2 get x's rows 0+1 and 2+3, rows 1 and 3 get y's rows 0+1 and 2+3.
template <int W>
__device__ inline float swap_add(float x, float y) {
    const unsigned ux = __float_as_uint(x), uy = __float_as_uint(y);
    const auto r = W == 32 ? __builtin_amdgcn_permlane32_swap(ux, uy, false, false)
                           : __builtin_amdgcn_permlane16_swap(ux, uy, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int NW, int TPW>
struct ScoreKernel {
    static constexpr int T = NW * TPW;
    static constexpr int NTHR = NW * 64;
    static constexpr int NCH = 1024 / NTHR;        // 16-byte chunks of a 64 x 128 fp16 tile per thread

    // one thread's share of a tile in flight; passed and returned by value so that it stays in registers
    struct TilePre {
        uint4 c[NCH];
    };
    __device__ static inline TilePre load_tile(const _Float16 *tiles, int kt, int tid) {
        const uint4 *src = reinterpret_cast<const uint4 *>(tiles) + (int64_t)kt * 1024;
        TilePre pf;
#pragma unroll
        for (int r = 0; r < NCH; ++r) pf.c[r] = src[tid + r * NTHR];
        return pf;
    }
    // registers -> LDS (padded rows), then a workgroup barrier: every thread calls it
    __device__ static inline void stage_tile(_Float16 *tile, int tid, const TilePre pf) {
#pragma unroll
        for (int r = 0; r < NCH; ++r) {
            const int c = tid + r * NTHR;
            *reinterpret_cast<uint4 *>(tile + (c >> 4) * SKS + (c & 15) * 8) = pf.c[r];
        }
        __syncthreads();
    }

    template <bool SEEDED>
    __device__ static inline void tile_mma(const half8 (&qf)[TPW][4], const _Float16 *tile, int lane,
                                           f32x4 (&acc)[TPW][4], const f32x4 (&seed)[TPW]) {
        const int n16 = lane & 15, g = lane >> 4;
        const _Float16 *bp = tile + n16 * SKS + g * 8;
        half8 b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)            // u -> (nt = u / 4, ks = u % 4)
            b[u] = *reinterpret_cast<const half8 *>(bp + (u >> 2) * 16 * SKS + (u & 3) * 32);
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            const int nt = u >> 2, ks = u & 3;
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                const f32x4 c0 = SEEDED ? seed[i] : f32x4{0.f, 0.f, 0.f, 0.f};
                acc[i][nt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(qf[i][ks], b[u & 3], ks == 0 ? c0 : acc[i][nt], 0, 0, 0);
            }
            if (u + 4 < 16) b[u & 3] = *reinterpret_cast<const half8 *>(bp + ((u + 4) >> 2) * 16 * SKS + ((u + 4) & 3) * 32);
        }
    }

    // POOL < 0: one output per compressed key.  POOL = 0 / 1: one output per selection block, the max over the
    // pooling window [4j - POOL, 4j - POOL + 5) of Eq. 6 (see vec2 below).
    template <int POOL>
    __device__ static void run(const ScoreArgs &a, int num_tiles) {
        extern __shared__ __attribute__((aligned(16))) _Float16 smem[];     // two tiles (double buffer)
        __shared__ int s_seq, s_tile, s_tbase[2];
        const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
        const int h = blockIdx.y;
        const int tile_id = num_tiles - 1 - (int)blockIdx.x;     // longest rows first
        if (tid == 0) {
            int rem = tile_id, s = 0, tb_fine = 0, tb_coarse = 0;      // first key tile of the sequence
            for (; s < a.map.batch; ++s) {
                const int slen = a.map.cu[s + 1] - a.map.cu[s];
                const int nt = (slen + T - 1) / T;
                if (rem < nt) break;
                rem -= nt;
                tb_fine += (num_cmp(slen, a.lc, a.sc) + kBlock - 1) / kBlock;
                tb_coarse += (num_cmp(slen, 4 * a.lc, 4 * a.sc) + kBlock - 1) / kBlock;
            }
            s_seq = s;
            s_tile = rem;
            s_tbase[0] = tb_fine;
            s_tbase[1] = tb_coarse;
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
        // this sequence's key tiles and their shifts (wave-uniform addresses)
        const int tb_fine = __builtin_amdgcn_readfirstlane(s_tbase[0]);
        const int tb_coarse = __builtin_amdgcn_readfirstlane(s_tbase[1]);
        const _Float16 *kt_fine = a.fine.data + ((int64_t)h * a.fine.tiles + tb_fine) * (kBlock * SD);
        const int32_t *sh_fine = a.fine.shift + (int64_t)h * a.fine.tiles + tb_fine;
        const _Float16 *kt_coarse = a.lse_mode ? a.coarse.data + ((int64_t)h * a.coarse.tiles + tb_coarse) * (kBlock * SD) : kt_fine;
        const int32_t *sh_coarse = a.lse_mode ? a.coarse.shift + (int64_t)h * a.coarse.tiles + tb_coarse : sh_fine;
        const int n16 = lane & 15, g = lane >> 4;

        // ---- Q rows of this wave's tokens: bf16 -> fp16, times a power of two (exact).  With
        // softmax_scale * log2(e) = cm * 2^ce (0.5 <= cm < 1), the keys carry cm (multiplied in when a tile is
        // converted to fp16) and the queries carry 2^ce, so the MFMA accumulator is the logit in the log2 domain.
        // A token whose magnitudes would leave fp16's comfortable range that way gets its own exponent instead and
        // takes the slower path that multiplies the accumulator by the difference.
        int ce;
        (void)frexpf(a.scale * S_LOG2E, &ce);
        half8 qf[TPW][4];
        int vis[TPW];
        // keys of pass 1: the fine ones, or with the LSE Approximation the coarse ones (Eq. 7)
        const int nc2 = num_cmp(len, 4 * a.lc, 4 * a.sc);
        int vis1[TPW];
        int vis1_min = 1 << 30;
        float cq[TPW];                   // 2^(ce - token's exponent): multiplies the accumulator (normally 1)
        bool q_plain = true;
        int vis_min = 1 << 30;
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            const int ti = w * TPW + i;
            vis[i] = ti < ntok ? min(visible_cmp(t0 + ti, a.lc, a.sc), nc) : 0;
            vis_min = min(vis_min, vis[i]);
            vis1[i] = a.lse_mode == 0 ? vis[i] : (ti < ntok ? min(visible_cmp(t0 + ti, 4 * a.lc, 4 * a.sc), nc2) : 0);
            vis1_min = min(vis1_min, vis1[i]);
            const uint16_t *qp = a.q + ((int64_t)(row0 + ti) * a.hq + h * SG + n16) * SD + g * 8;
            float x[4][8];
            float amax = 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const uint4 raw = ti < ntok ? *reinterpret_cast<const uint4 *>(qp + ks * 32) : make_uint4(0, 0, 0, 0);
                const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    x[ks][2 * e] = __uint_as_float(u[e] << 16);
                    x[ks][2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
                    amax = fmaxf(amax, fmaxf(fabsf(x[ks][2 * e]), fabsf(x[ks][2 * e + 1])));
                }
            }
            amax = wave_max(amax);
            if (!(amax < 3.0e38f)) amax = 3.0e38f;     // Inf / NaN inputs: keep going, results are Inf / NaN anyway
            int exq = 0;
            if (amax > 0.f) (void)frexpf(amax, &exq);  // amax = f * 2^exq, 0.5 <= f < 1
            // keep the largest magnitude within [2^-8, 2^15): 18+ binades of full precision below it
            int eq = ce;
            if (exq + ce > 15 || exq + ce < -8) eq = 4 - exq;
            const float sc = __builtin_ldexpf(1.0f, eq);
            cq[i] = __builtin_ldexpf(1.0f, ce - eq);
            q_plain &= eq == ce;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int e = 0; e < 8; ++e) qf[i][ks][e] = (_Float16)(x[ks][e] * sc);
        }
        f32x4 acc[TPW][4];
        f32x4 nm[TPW];                   // per lane and head row: minus the reference (log2 domain)
        float l[TPW][4];                 // ... and the sum of 2^(y - reference)
#pragma unroll
        for (int i = 0; i < TPW; ++i) {
            nm[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < 4; ++r) l[i][r] = 0.f;
        }

        // Matrix-core step of either pass: acc = y - seed for tile kt (y = the logit in the log2 domain)
        auto mma = [&](int kt, const int32_t *shifts, const f32x4 (&seed)[TPW]) {
            const _Float16 *tile = smem + (kt & 1) * S_TILE;
            const int tshift = shifts[kt];
            if (q_plain && tshift == 0) {
                tile_mma<true>(qf, tile, lane, acc, seed);
            } else {
                tile_mma<false>(qf, tile, lane, acc, seed);
                const float tsc = __builtin_ldexpf(1.0f, tshift);
#pragma unroll
                for (int i = 0; i < TPW; ++i)
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) acc[i][nt][r] = __builtin_fmaf(acc[i][nt][r], cq[i] * tsc, seed[i][r]);
            }
        };
        // The two waves that share a SIMD (w and w + NW/2) run half a step apart: between two barriers the first
        // does the matrix-core step of tile kt and then its vector step, the second does the vector step of tile
        // kt - 1 (still in its accumulators) and then the matrix-core step of tile kt.  Matrix core and vector
        // unit of a SIMD are then busy at the same time although each wave alternates between them.
        const bool late = w >= NW / 2;

        // ------------------------------------------------ pass 1: log-sum-exp of every (token, head) row
        // First attempt without a running reference: sum 2^y as it is.  For ordinary activations |y| stays far
        // below fp32's exponent range, and the max tracking (a fifth of the vector work of this pass) is saved.
        // If any row's sum then overflowed, vanished or is NaN, the workgroup repeats the pass with the reference.
        auto vec1 = [&](int kt, auto tracked_c) {
            constexpr bool tracked = decltype(tracked_c)::value;
            const int kbase = kt * kBlock;
            const bool edge_tile = kbase + kBlock > vis1_min;
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                if (edge_tile) {
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt)
                        if (kbase + nt * 16 + n16 >= vis1[i]) acc[i][nt] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
                }
                // The reference moves only when an exponent exceeds S_SLACK; the first tile sets it (up or down).
                if (tracked) {
                    float mx[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) mx[r] = fmaxf(fmaxf(acc[i][0][r], acc[i][1][r]), fmaxf(acc[i][2][r], acc[i][3][r]));
                    const float mxall = fmaxf(fmaxf(mx[0], mx[1]), fmaxf(mx[2], mx[3]));
                    if (kt == 0 || __any(mxall > S_SLACK)) {
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            float d = kt == 0 ? mx[r] : fmaxf(mx[r], 0.f);
                            if (!(d > -3.0e38f)) d = 0.f;              // nothing visible in this lane's columns yet
                            l[i][r] *= s_exp2(-d);
                            nm[i][r] -= d;
#pragma unroll
                            for (int nt = 0; nt < 4; ++nt) acc[i][nt][r] -= d;
                        }
                    }
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float sum = l[i][r];
#pragma unroll
                    for (int nt = 0; nt < 4; ++nt) sum += s_exp2(acc[i][nt][r]);
                    l[i][r] = sum;
                }
            }
        };
        const int vis1_last = a.lse_mode == 0 ? vis_last : min(visible_cmp(t0 + ntok - 1, 4 * a.lc, 4 * a.sc), nc2);
        const int nkt1 = (vis1_last + kBlock - 1) / kBlock;
        float lse2[TPW][4];
        auto pass1 = [&](auto tracked_c) -> bool {       // returns true if some row's sum cannot be trusted
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                nm[i] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int r = 0; r < 4; ++r) l[i][r] = 0.f;
            }
            TilePre pf = {};
            if (nkt1 > 0) stage_tile(smem, tid, load_tile(kt_coarse, 0, tid));
            for (int kt = 0; kt < nkt1; ++kt) {
                if (kt + 1 < nkt1) pf = load_tile(kt_coarse, kt + 1, tid);
                if (late && kt > 0) vec1(kt - 1, tracked_c);
                mma(kt, sh_coarse, nm);
                if (!late) vec1(kt, tracked_c);
                if (kt + 1 < nkt1) stage_tile(smem + ((kt + 1) & 1) * S_TILE, tid, pf);
                else __syncthreads();
            }
            if (late && nkt1 > 0) vec1(nkt1 - 1, tracked_c);
            // merge the 16 key lanes of each lane group; lse2 = log2 of the row's sum of 2^y
            bool bad = false;
#pragma unroll
            for (int i = 0; i < TPW; ++i)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    // (lane moves inside the 16-lane row: no LDS round trips)
                    float mm = -nm[i][r], ll = l[i][r];
                    const float mrow = row16_all<true>(mm);
                    ll = row16_all<false>(ll * s_exp2(mm - mrow));
                    mm = mrow;
                    // a row that saw no key at all (possible with the coarse keys of the LSE Approximation while
                    // fine keys are already visible) normalises everything to zero
                    lse2[i][r] = ll > 0.f ? mm + __log2f(ll) : INFINITY;
                    // untracked sums are trusted only well inside fp32's range (2^-64 .. 3e38)
                    bad |= vis1[i] > 0 && !(ll >= 5.4e-20f && ll < 3.0e38f);
                }
            return bad;
        };
        if (__syncthreads_or(pass1(std::false_type{}))) (void)pass1(std::true_type{});

        // ------------------------------------------------ pass 2: normalised scores, group sum, store
        f32x4 nlse[TPW];
#pragma unroll
        for (int i = 0; i < TPW; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) nlse[i][r] = -lse2[i][r];
        // Fused pooling (POOL >= 0).  After the butterfly lane x of the wave holds the group sum of key kbase + x,
        // so the four keys 4m .. 4m + 3 of the tile sit in one lane quad and their max takes two quad swaps.  The
        // fifth key of a window lies one lane below the quad (POOL = 1: window = key 4m - 1 and quad m, block
        // 16 kt + m) or is the first lane of the next quad (POOL = 0: window = quad m - 1 and key 4m, block
        // 16 kt + m - 1): either way lane 4m combines its own value with one shifted up by a lane, and what
        // lane 0 needs from the previous tile of the same token is carried in a scalar.
        unsigned carry[TPW];                 // bit patterns of non-negative floats
#pragma unroll
        for (int i = 0; i < TPW; ++i) carry[i] = 0u;
        float *const out_w = a.out + ((int64_t)h * a.map.total_rows + row0 + w * TPW) * a.row_stride;
        auto vec2_body = [&](int kt, auto edge_c) {
            constexpr bool edge_tile = decltype(edge_c)::value;   // the tile reaches past some token's visible keys
            const int kbase = kt * kBlock;
            const int jb = kt * (kBlock / 4) + (lane >> 2) - (POOL > 0 ? 0 : 1);     // the block lane 4m completes
            const bool writer = (lane & 3) == 0 && jb >= 0;
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                float s[4];
#pragma unroll
                for (int nt = 0; nt < 4; ++nt)
                    s[nt] = (s_exp2(acc[i][nt][0]) + s_exp2(acc[i][nt][1])) + (s_exp2(acc[i][nt][2]) + s_exp2(acc[i][nt][3]));
                // butterfly over the four lane groups: afterwards lane (n16, g) holds n-tile g, i.e. key kbase + lane
                // (a half swap of (s0, s2) and of (s1, s3), then a row swap of the two sums: no LDS round trip)
                const float a0 = swap_add<32>(s[0], s[2]);
                const float a1 = swap_add<32>(s[1], s[3]);
                const float f = swap_add<16>(a0, a1);
                const int key = kbase + lane;
                if (POOL < 0) {
                    if (key < vis[i]) out_w[i * a.row_stride + key] = f;
                } else {
                    // scores are >= 0: an invisible key counts as 0, and the maxima are taken on the bit patterns
                    // (same order as the floats; an integer max folds the lane move into itself)
                    const unsigned fz = edge_tile && key >= vis[i] ? 0u : __float_as_uint(f);
                    unsigned qm = max(fz, dpp_move<DPP_QUAD_SWAP1>(fz));
                    qm = max(qm, dpp_move<DPP_QUAD_SWAP2>(qm));
                    const unsigned shifted_src = POOL ? fz : qm, own = POOL ? qm : fz;
                    unsigned below = dpp_move<DPP_WAVE_SHR1>(shifted_src);
                    if (lane == 0) below = carry[i];
                    carry[i] = __builtin_amdgcn_readlane(shifted_src, 63);
                    const bool has_visible_key = !edge_tile || max(4 * jb - POOL, 0) < vis[i];
                    if (writer && has_visible_key) out_w[i * a.row_stride + jb] = __uint_as_float(max(below, own));
                }
            }
        };
        auto vec2 = [&](int kt) {
            // only tiles that reach past the visible prefix of one of the wave's tokens need per-lane checks
            if (POOL < 0 || kt * kBlock + kBlock > vis_min) vec2_body(kt, std::true_type{});
            else vec2_body(kt, std::false_type{});
        };
        // the block whose window starts in the last tile but would end in the next one
        auto flush_pool = [&]() {
            if (POOL < 0) return;
            const int jb = nkt * (kBlock / 4) - (POOL ? 0 : 1);
#pragma unroll
            for (int i = 0; i < TPW; ++i)
                if (lane == 0 && max(4 * jb - POOL, 0) < vis[i]) out_w[i * a.row_stride + jb] = __uint_as_float(carry[i]);
        };
        TilePre pf = load_tile(kt_fine, 0, tid);
        stage_tile(smem, tid, pf);
        for (int kt = 0; kt < nkt; ++kt) {
            if (kt + 1 < nkt) pf = load_tile(kt_fine, kt + 1, tid);
            if (late && kt > 0) vec2(kt - 1);
            mma(kt, sh_fine, nlse);
            if (!late) vec2(kt);
            if (kt + 1 < nkt) stage_tile(smem + ((kt + 1) & 1) * S_TILE, tid, pf);
            else __syncthreads();
        }
        if (late) vec2(nkt - 1);
        flush_pool();
    }
};

template <int NW, int TPW, int POOL>
__global__ void __launch_bounds__(NW * 64) block_scores_mfma_kernel(ScoreArgs a, int num_tiles) {
    ScoreKernel<NW, TPW>::template run<POOL>(a, num_tiles);
}

template <int NW, int TPW, int POOL>
int launch_scores_mfma(const Launch &L, ScoreArgs a, const int32_t *cu_h) {
    constexpr int T = NW * TPW;
    int64_t tiles = 0, kt_fine = 0, kt_coarse = 0;
    for (int s = 0; s < L.map.batch; ++s) {
        const int len = cu_h[s + 1] - cu_h[s];
        tiles += (len + T - 1) / T;
        kt_fine += (num_cmp(len, a.lc, a.sc) + kBlock - 1) / kBlock;
        if (a.lse_mode) kt_coarse += (num_cmp(len, 4 * a.lc, 4 * a.sc) + kBlock - 1) / kBlock;
    }
    if (tiles == 0 || kt_fine == 0) return INFLLMV2_OK;      // no token sees a compressed key
    if (kt_fine + kt_coarse > 0x7fffffff) return INFLLMV2_ERR_UNSUPPORTED;
    // fp16 key tiles + one shift per tile, in the caller's workspace
    const int hkv = L.p->num_kv_heads;
    const size_t tile_bytes = (size_t)kBlock * SD * sizeof(_Float16);
    const size_t data_bytes = (size_t)hkv * (kt_fine + kt_coarse) * tile_bytes;
    const size_t ws_bytes = data_bytes + (size_t)hkv * (kt_fine + kt_coarse) * sizeof(int32_t);
    void *ws = L.ws;
    if (ws == nullptr || L.ws_bytes < ws_bytes) return INFLLMV2_ERR_WORKSPACE_TOO_SMALL;
    _Float16 *fine = (_Float16 *)ws, *coarse = fine + (size_t)hkv * kt_fine * kBlock * SD;
    int32_t *sh_fine = (int32_t *)((char *)ws + data_bytes), *sh_coarse = sh_fine + (size_t)hkv * kt_fine;
    int ce;
    const float cm = frexpf(a.scale * S_LOG2E, &ce);
    hipLaunchKernelGGL(kc_half_kernel, dim3((unsigned)(kt_fine + kt_coarse), hkv), dim3(256), 0, L.stream, a.kc, L.map,
                       a.lc, a.sc, a.dense_below, cm, fine, sh_fine, (int)kt_fine, coarse, sh_coarse, (int)kt_coarse);
    a.fine = HalfTiles{fine, sh_fine, (int32_t)kt_fine};
    a.coarse = HalfTiles{coarse, sh_coarse, (int32_t)kt_coarse};
    const size_t lds = (size_t)2 * S_TILE * sizeof(_Float16);
    dim3 grid((unsigned)tiles, hkv);
    hipLaunchKernelGGL((block_scores_mfma_kernel<NW, TPW, POOL>), grid, dim3(NW * 64), lds, L.stream, a, (int)tiles);
    return hip_status(hipGetLastError());
}

bool scores_mfma_params(const infllmv2_params *p, bool pooled) {
    // the tiled kernel pools on chip only for the paper's window (l = 5, s = 4), unshifted or shifted by one, with
    // four compressed keys per selection block (block j's window then starts at key 4j of its tile row)
    const bool pool_ok = !pooled || (p->pool_len == 5 && p->pool_stride == 4 && (p->pool_pad == 0 || p->pool_pad == 1) &&
                                     p->cmp_stride * p->pool_stride == kBlock);
    return p->dtype == INFLLMV2_BF16 && p->head_dim == SD && p->num_q_heads / p->num_kv_heads == SG && pool_ok;
}

}  // namespace

// fp16 copies of the fine (and, with the LSE Approximation, coarse) key tiles plus one shift per tile
size_t scores_ws_bytes(const infllmv2_params *p, const BatchTotals &t, bool pooled) {
    if (!scores_mfma_params(p, pooled)) return 0;
    const int64_t tiles = t.kt_fine + (p->lse_mode ? t.kt_coarse : 0);
    return align256((size_t)p->num_kv_heads * tiles * ((size_t)kBlock * SD * sizeof(_Float16) + sizeof(int32_t)));
}

int launch_block_scores(const Launch &L, const void *q, const float *kc, float *s_shared, int64_t row_stride,
                        const int32_t *cu_h, bool pooled) {
    const bool bf = L.p->dtype == INFLLMV2_BF16;
    const PoolArgs pool{pooled ? 1 : 0, L.p->pool_len, L.p->pool_stride, L.p->pool_pad};
    if (cu_h != nullptr && L.map.ctx == nullptr && scores_mfma_params(L.p, pooled) &&
        (((uintptr_t)q | (uintptr_t)kc) & 15) == 0) {
        ScoreArgs a{(const uint16_t *)q, kc, HalfTiles{}, HalfTiles{}, s_shared, L.map, L.p->num_q_heads, L.p->cmp_len, L.p->cmp_stride,
                    L.p->dense_threshold, L.p->lse_mode, L.p->softmax_scale, row_stride};
        if (!pooled) return launch_scores_mfma<8, 4, -1>(L, a, cu_h);
        return pool.pad == 0 ? launch_scores_mfma<8, 4, 0>(L, a, cu_h) : launch_scores_mfma<8, 4, 1>(L, a, cu_h);
    }
    if (L.p->head_dim == 128)
        return bf ? launch_generic<bf16_t, 128>(L, q, kc, s_shared, row_stride, pool)
                  : launch_generic<float, 128>(L, q, kc, s_shared, row_stride, pool);
    return bf ? launch_generic<bf16_t, 64>(L, q, kc, s_shared, row_stride, pool)
              : launch_generic<float, 64>(L, q, kc, s_shared, row_stride, pool);
}

}  // namespace ifv2
