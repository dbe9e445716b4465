// Decode step for bf16 caches, G = 16, d_h = 128: stages 2-4 of the method for the single query row
// t = L-1 of every sequence (the row of Alg. 1 / Eq. 2 / Alg. 2 that a prefill would compute last).
// The step moves ~100 MB (compressed-key cache once, 64 selected K/V blocks per KV head) and does almost no
// arithmetic, so the work of one (sequence, KV head) pair is split over many workgroups to fill the chip;
// reductions that need a whole pair sit behind kernel boundaries.  A kernel boundary is the cheap way to make one
// workgroup's results visible to another on a multi-die GPU: letting the last attend workgroup of a pair do the
// merge (device-wide fence + counter) was measured slower than the extra launch, 58.6 vs 53.3 us, because the
// fences act on whole caches.
//
// Two forms.  With the exact normalisation (lse_mode 0) the step is front / pool / attend / merge, described at the
// kernels ("three-stage form" below): the blocks Eq. 2 always keeps are attended beside the score computation,
// normalisation and max-pooling are spread over many workgroups, and the selection itself is repeated by each
// attend workgroup, so no kernel of the chain works through a pair alone.  With the LSE Approximation (Sec. 3.4) it
// is the older chain
//   scores  : grid (key chunks, pairs)  logits of 128 compressed keys x 16 heads per workgroup, written once
//             as log2-domain logits, plus per-chunk (max, sum) partials of the softmax normaliser
//   select  : grid (pairs)              one 1024-thread workgroup per pair forms the normaliser from means of four
//             logits (the coarse keys' logits), sums the normalised scores of the 16 heads (Eq. 5) into LDS,
//             max-pools them to blocks (Eq. 6) and selects (Eq. 2) with a workgroup-wide radix select.  The score
//             row of a pair must fit in LDS (contexts up to ~419K tokens).
//   attend  : grid (splits, pairs)      one wavefront per selected block: K fragments straight from global
//             memory into MFMA operands, V through a 16 KB LDS tile (MFMA unit shared with prefill); the
//             eight partial results of a workgroup are merged in LDS
//   merge   : grid (pairs)              log-sum-exp merge of the per-split partial outputs, writes O and lse
// K^{C1} is float32; it is split into a bf16 high part and a bf16 residual in registers and both products
// are accumulated, so the logits carry ~16 mantissa bits of K^{C1}.
#include "attn_unit.h"
#include "topk_row.h"

namespace ifv2 {

namespace {

using namespace attn_unit;

constexpr int SC_TILES = 2;               // 16-key tiles per wave of the scores kernel
constexpr int CK = 4 * SC_TILES * 16;     // compressed keys per scores workgroup (4 waves)
constexpr int OPART = G * D;      // floats of one partial output

struct DecArgs {
    const uint16_t *q, *k, *v;
    const float *kc;
    const int32_t *ctx;
    int batch, hkv, hq;
    int64_t kv_batch_stride, kv_head_stride, kv_tok_stride, kc_head_stride;
    float scale;
    TopkArgs tk;
    float *z;          // [pairs][zs keys][16 heads] log2-domain logits c * <q, kc>
    float *part;       // [pairs][nchunk][16][2] (max, sum 2^(z - max)) per chunk
    int32_t *idx;      // [pairs][topk_total]
    float *opart;      // [pairs][nsplit][OPART]  partial O^T relative to the split's own max, in the attend kernel's
                       // register order: float4 slot dt * 64 + lane = dims 16 dt + 4 (lane / 16) .. + 3 of head lane % 16
    float *mlpart;     // [pairs][nsplit][16][2]
    uint16_t *out;     // [batch][hq][d]
    float *lse;        // [batch][hq] or nullptr
    int zs, nchunk, nsplit;
    int lse_mode;      // 1: normalise with the log-sum-exp over the four times coarser keys (LSE Approximation, Sec. 3.4)
    // three-stage form (front / pool / attend + merge):
    uint32_t *pk;      // [pairs][pk_cap] pooled score of every block (bit pattern of a float >= 0; 0 for forced blocks)
    int pk_cap;
    int fsplit;        // partial-output slots taken by the forced blocks (attended beside the scores)
    int nslot;         // fsplit + nsplit
    int bpw;           // blocks per attend workgroup (<= its number of waves): list entries split * bpw .. + bpw - 1
};

// Which blocks the newest token of an L-token sequence always keeps (Eq. 2: the first n_init and the last n_local
// blocks), and how many of the others the top-k adds.
struct Forced {
    int bt, nblk, f_init, f_lo, n_forced, n_rest, kr;
    __host__ __device__ Forced(const TopkArgs &tk, int L) {
        bt = (L - 1) / kBlock;
        nblk = bt + 1;
        f_init = tk.n_init < nblk ? tk.n_init : nblk;
        f_lo = bt - tk.n_local + 1 > 0 ? bt - tk.n_local + 1 : 0;
        n_forced = f_init + (bt - f_lo + 1) - (f_init > f_lo ? f_init - f_lo : 0);
        n_rest = nblk - n_forced;
        const int want = tk.topk_total - tk.n_init - tk.n_local;
        kr = want < n_rest ? want : n_rest;
    }
    // e-th forced block in ascending order, e < n_forced
    __host__ __device__ int forced_block(int e) const { return e < f_init ? e : (f_lo > f_init ? f_lo : f_init) + (e - f_init); }
    __host__ __device__ bool is_forced(int j) const { return j < f_init || j >= f_lo; }
};

// reductions over the 16 lanes of a row (lanes with equal lane / 16), result in every lane, without LDS: swaps inside
// quads, then the mirror images inside 8 and 16 lanes
template <int CTRL>
__device__ inline float row_move(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
__device__ inline float row_all_max(float x) {
    x = fmaxf(x, row_move<0xB1>(x));      // quad_perm [1,0,3,2]
    x = fmaxf(x, row_move<0x4E>(x));      // quad_perm [2,3,0,1]
    x = fmaxf(x, row_move<0x141>(x));     // row_half_mirror
    return fmaxf(x, row_move<0x140>(x));  // row_mirror
}
__device__ inline float row_all_sum(float x) {
    x += row_move<0xB1>(x);
    x += row_move<0x4E>(x);
    x += row_move<0x141>(x);
    return x + row_move<0x140>(x);
}

// sum over the four 16-lane rows of a wave (lanes with equal lane % 16), result in every lane
__device__ inline float rows_sum(float x) {
    const unsigned u = __float_as_uint(x);
    const auto p = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const float s1 = __uint_as_float(p[0]) + __uint_as_float(p[1]);
    const unsigned v = __float_as_uint(s1);
    const auto q = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// inclusive prefix sum over the 64 lanes of a wave in lane order, without LDS: shifts inside the 16-lane rows, then
// the last lane of a row broadcast into the next row(s)
__device__ inline int wave_inclusive_sum(int x) {
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, true);      // row_shr:1 (zero shifted in)
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, true);      // row_shr:2
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, true);      // row_shr:4
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, true);      // row_shr:8
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, false);     // row_bcast:15 into rows 1 and 3
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, false);     // row_bcast:31 into rows 2 and 3
    return x;
}

// ------------------------------------------------------------------------------------------ scores
__device__ inline void score_chunk(const DecArgs &a, int chunk, int pair) {
    const int b = pair / a.hkv, h = pair - b * a.hkv;
    const int L = a.ctx[b];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int n16 = lane & 15, g = lane >> 4;
    __shared__ float red[4][16][2];
    float *part = a.part + ((int64_t)pair * a.nchunk + chunk) * 32;
    const bool dense = L < a.tk.dense_below;
    const int v = dense ? 0 : visible_cmp(L - 1, a.tk.lc, a.tk.sc);
    const float c = a.scale * LOG2E;
    if (chunk * CK >= v) {                       // nothing visible here (or a dense sequence)
        if (tid < 16) { part[tid * 2] = -INFINITY; part[tid * 2 + 1] = 0.f; }
    } else {
        const uint16_t *qp = a.q + ((int64_t)b * a.hq + h * G + n16) * D + g * 8;
        bf16x8 qf[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) qf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(qp + s * 32));
        const float *kcb = a.kc + (int64_t)pair * a.kc_head_stride;
        // every load of the wave is requested before anything is computed: one trip to memory, not one per tile
        float4 xs[SC_TILES][4][2];
#pragma unroll
        for (int nt = 0; nt < SC_TILES; ++nt) {
            const int key = chunk * CK + w * (SC_TILES * 16) + nt * 16 + n16;
            const float *kr = kcb + (int64_t)(key < v ? key : 0) * D + g * 8;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                xs[nt][s][0] = *reinterpret_cast<const float4 *>(kr + s * 32);
                xs[nt][s][1] = *reinterpret_cast<const float4 *>(kr + s * 32 + 4);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        float zc[SC_TILES][4];                         // logits of key tile nt, heads 4g .. 4g+3 (-inf: not visible)
#pragma unroll
        for (int nt = 0; nt < SC_TILES; ++nt) {
            const int key = chunk * CK + w * (SC_TILES * 16) + nt * 16 + n16;
            const bool valid = key < v;
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const float4 x0 = xs[nt][s][0], x1 = xs[nt][s][1];
                const float x[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
                bf16x8 bh, bl;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const __bf16 hi = (__bf16)x[e];
                    bh[e] = hi;
                    bl[e] = (__bf16)(x[e] - (float)hi);
                }
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[s], bh, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[s], bl, acc, 0, 0, 0);
            }
            // acc[r] = <q_head(4g+r), kc_key>: the key's 16 logits are 64 contiguous bytes, this lane writes 16 of them
            const float4 zv = make_float4(acc[0] * c, acc[1] * c, acc[2] * c, acc[3] * c);
            if (valid) *reinterpret_cast<float4 *>(a.z + ((int64_t)pair * a.zs + key) * G + 4 * g) = zv;
            zc[nt][0] = valid ? zv.x : -INFINITY;
            zc[nt][1] = valid ? zv.y : -INFINITY;
            zc[nt][2] = valid ? zv.z : -INFINITY;
            zc[nt][3] = valid ? zv.w : -INFINITY;
        }
        // per head: max and sum of 2^(z - max) over the wave's keys -- over this lane's tiles, then over the 16 key
        // lanes with data-parallel moves (no LDS round trips)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float mm = zc[0][r];
#pragma unroll
            for (int nt = 1; nt < SC_TILES; ++nt) mm = fmaxf(mm, zc[nt][r]);
            mm = row_all_max(mm);
            const float ms = mm == -INFINITY ? 0.f : mm;
            float ll = 0.f;
#pragma unroll
            for (int nt = 0; nt < SC_TILES; ++nt) ll += fast_exp2(zc[nt][r] - ms);
            ll = row_all_sum(ll);
            if (n16 == 0) { red[w][4 * g + r][0] = mm; red[w][4 * g + r][1] = ll; }
        }
        __syncthreads();
        if (tid < 16) {
            float mm = -INFINITY;
            for (int k = 0; k < 4; ++k) mm = fmaxf(mm, red[k][tid][0]);
            float ll = 0.f;
            for (int k = 0; k < 4; ++k)
                if (red[k][tid][0] != -INFINITY) ll += red[k][tid][1] * fast_exp2(red[k][tid][0] - mm);
            part[tid * 2] = mm;
            part[tid * 2 + 1] = ll;
        }
    }
}

__global__ void __launch_bounds__(256) dec_scores_kernel(DecArgs a) { score_chunk(a, blockIdx.x, blockIdx.y); }

// ------------------------------------------------------------------------------------------ select
// Stages 2b-3 for one (sequence, KV head) pair in one workgroup.  Selection rule and tie handling are those of
// topk_row: keys above the k-th largest, then the first `need` keys equal to it in ascending block order.
constexpr int SEL_THREADS = 1024;
constexpr size_t kSelLdsMax = 128 * 1024;     // dynamic LDS of the select kernel: score row + pooled keys
constexpr int SEL_WAVES = SEL_THREADS / 64;

// exclusive prefix count of `flag` over the workgroup's threads in thread order (+ total); two barriers
__device__ inline int wg_prefix_count(bool flag, int *wave_tot, int tid, int &total) {
    const int lane = tid & 63, w = tid >> 6;
    const uint64_t b = __ballot(flag);
    const int within = __popcll(b & ((1ull << lane) - 1ull));
    __syncthreads();                                   // previous readers of wave_tot are done
    if (lane == 0) wave_tot[w] = __popcll(b);
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int k = 0; k < SEL_WAVES; ++k) {
        const int t = wave_tot[k];
        before += k < w ? t : 0;
        tot += t;
    }
    total = tot;
    return before + within;
}

__global__ void __launch_bounds__(SEL_THREADS) dec_select_kernel(DecArgs a, int sh_cap) {
    extern __shared__ __attribute__((aligned(16))) float sel_smem[];
    float *sh = sel_smem;                                              // [sh_cap] group scores of the row
    uint32_t *pk = reinterpret_cast<uint32_t *>(sel_smem + sh_cap);    // [blocks of the longest context + 4] pooled keys
    __shared__ float red[64][16][2];
    __shared__ float lse2[16];
    __shared__ int hist[4][256];                 // one histogram per radix pass, all zeroed up front
    __shared__ int wave_tot[SEL_WAVES];
    __shared__ uint32_t s_prefix;
    __shared__ int s_k;
    const int pair = blockIdx.x;
    const int b = pair / a.hkv;
    const int L = a.ctx[b];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    int32_t *out = a.idx + (int64_t)pair * a.tk.topk_total;
    if (L < a.tk.dense_below) {                      // dense sequences attend to every block: no list
        for (int j = tid; j < a.tk.topk_total; j += SEL_THREADS) out[j] = -1;
        return;
    }
    const int t = L - 1;
    const int v = visible_cmp(t, a.tk.lc, a.tk.sc);
    const int bt = t / kBlock, nblk = bt + 1;
    // forced blocks: [0, n_init) and (bt - n_local, bt]
    const int f_init = min(a.tk.n_init, nblk);
    const int f_lo = max(0, bt - a.tk.n_local + 1);
    const int n_forced = f_init + (bt - f_lo + 1) - max(0, f_init - f_lo);
    const int n_rest = nblk - n_forced;
    const int kr = min(a.tk.topk_total - a.tk.n_init - a.tk.n_local, n_rest);
    if (kr == n_rest) {                              // everything up to the query's block is kept
        for (int j = tid; j < a.tk.topk_total; j += SEL_THREADS) out[j] = j < nblk ? j : -1;
        return;
    }
    // The logits this thread will normalise (up to ZPT keys x 16 heads) are requested first, so that their trip to
    // memory overlaps the merge of the normaliser below.
    constexpr int ZPT = 4;                               // covers 4096 compressed keys = 65K tokens of context
    float zr[ZPT][G];
    {
        const float *zb0 = a.z + (int64_t)pair * a.zs * G;
#pragma unroll
        for (int u = 0; u < ZPT; ++u) {
            const int i = min(tid + u * SEL_THREADS, max(v - 1, 0));
            const float4 *zk = reinterpret_cast<const float4 *>(zb0 + (int64_t)i * G);
#pragma unroll
            for (int q4 = 0; q4 < G / 4; ++q4) {
                const float4 t4 = zk[q4];
                zr[u][4 * q4] = t4.x; zr[u][4 * q4 + 1] = t4.y; zr[u][4 * q4 + 2] = t4.z; zr[u][4 * q4 + 3] = t4.w;
            }
        }
    }
    // ---- log2 of sum_i 2^z per head: 64 thread groups per head over the chunk partials, then 64 -> 1
    if (a.lse_mode == 0) {
        const int head = tid & 15, pg = tid >> 4;
        const float *pp = a.part + (int64_t)pair * a.nchunk * 32 + head * 2;
        float mm = -INFINITY, ll = 0.f;
        for (int ch = pg; ch < a.nchunk; ch += 64) {
            const float mo = pp[ch * 32], lo = pp[ch * 32 + 1];
            const float mn = fmaxf(mm, mo);
            const float ms = mn == -INFINITY ? 0.f : mn;
            ll = ll * fast_exp2(mm - ms) + lo * fast_exp2(mo - ms);
            mm = mn;
        }
        red[pg][head][0] = mm;
        red[pg][head][1] = ll;
    } else {
        // LSE Approximation (Eq. 7): the normaliser runs over the coarse keys.  K^{C2}_i is the mean of the four
        // disjoint K^{C1} windows 4i + m l/s, m = 0..3, and the logit is linear in the key, so the coarse logit is
        // the mean of four logits already in z -- no second product.  Thread groups as above, over coarse keys.
        const int head = tid & 15, pg = tid >> 4;
        const int cstep = a.tk.lc / a.tk.sc;
        const int v2 = min(visible_cmp(t, 4 * a.tk.lc, 4 * a.tk.sc), num_cmp(L, 4 * a.tk.lc, 4 * a.tk.sc));
        const float *zh = a.z + (int64_t)pair * a.zs * G + head;           // logit of key i at zh[i * G]
        float mm = -INFINITY, ll = 0.f;
        for (int i2 = pg; i2 < v2; i2 += 64) {
            const float zc = 0.25f * ((zh[(4 * i2) * G] + zh[(4 * i2 + cstep) * G]) +
                                      (zh[(4 * i2 + 2 * cstep) * G] + zh[(4 * i2 + 3 * cstep) * G]));
            const float mn = fmaxf(mm, zc);
            ll = ll * fast_exp2(mm - mn) + fast_exp2(zc - mn);
            mm = mn;
        }
        red[pg][head][0] = mm;
        red[pg][head][1] = ll;
    }
    {
        // 64 -> 1 per head: wavefront w takes head w, one thread group per lane, merged with lane moves
        __syncthreads();
        static_assert(SEL_WAVES == G, "one wavefront per head");
        const float mk = red[lane][w][0], lk = red[lane][w][1];
        const float m2 = rows_max(row_all_max(mk));
        const float l2 = rows_sum(row_all_sum(mk == -INFINITY ? 0.f : lk * fast_exp2(mk - m2)));
        // no coarse key visible yet (LSE Approximation only): every score is zero
        if (lane == 0) lse2[w] = l2 > 0.f ? m2 + __log2f(l2) : INFINITY;
        __syncthreads();
    }
    // ---- S^shared[i] = sum over the 16 heads of 2^(z[g][i] - lse2[g]), kept in LDS
#pragma unroll
    for (int u = 0; u < ZPT; ++u) {
        const int i = tid + u * SEL_THREADS;
        if (i < v) {
            float sum = 0.f;
#pragma unroll
            for (int gq = 0; gq < G; ++gq) sum += fast_exp2(zr[u][gq] - lse2[gq]);
            sh[i] = sum;
        }
    }
    for (int i = tid + ZPT * SEL_THREADS; i < v; i += SEL_THREADS) {      // longer contexts: the rest, unprefetched
        const float *zb = a.z + ((int64_t)pair * a.zs + i) * G;
        float sum = 0.f;
#pragma unroll
        for (int gq = 0; gq < G; ++gq) sum += fast_exp2(zb[gq] - lse2[gq]);
        sh[i] = sum;
    }
    __syncthreads();
    // ---- pooled key of every block (0 for forced blocks: they take no part in the top-k)
    auto live = [&](int j) -> bool { return j < nblk && !(j < f_init || j >= f_lo); };
    for (int j = tid; j < nblk; j += SEL_THREADS) {
        float m = 0.f;
        if (live(j)) {
            const int lo = a.tk.pool_stride * j - a.tk.pool_pad;
            for (int u = 0; u < a.tk.pool_len; ++u) {
                const int i = lo + u;
                if (i >= 0 && i < v) m = fmaxf(m, sh[i]);
            }
        }
        pk[j] = __float_as_uint(m);
    }
    if (tid == 0) { s_prefix = 0u; s_k = kr; }
    (&hist[0][0])[tid] = 0;                      // SEL_THREADS = 4 x 256
    __syncthreads();
    // ---- radix select (4 x 8 bits) of the kr-th largest key among the live blocks
    static_assert(SEL_THREADS == 4 * 256, "histograms zeroed by one store per thread");
    for (int pass = 3; pass >= 0; --pass) {
        const uint32_t prefix = s_prefix;
        const int hi_shift = 8 * (pass + 1);
        for (int j = tid; j < nblk; j += SEL_THREADS) {
            if (!live(j)) continue;
            const uint32_t key = pk[j];
            if (pass == 3 || (key >> hi_shift) == prefix) atomicAdd(&hist[pass][(key >> (8 * pass)) & 255u], 1);
        }
        __syncthreads();
        if (w == 0) {
            // lane l owns digits 4l .. 4l+3; above[d] = number of keys with a larger digit
            const int k = s_k;
            int c[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) c[u] = hist[pass][4 * lane + u];
            const int mine = c[0] + c[1] + c[2] + c[3];
            int higher = 0;                              // keys in lanes above this one
            {
                int run = mine;                          // inclusive suffix sum over lanes
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const int other = __shfl_down(run, o);
                    if (lane + o < 64) run += other;
                }
                higher = run - mine;
            }
            int above = higher;
#pragma unroll
            for (int u = 3; u >= 0; --u) {
                // digit d = 4 lane + u holds the k-th largest iff above < k <= above + c[u]
                if (above < k && k <= above + c[u]) {
                    s_prefix = (prefix << 8) | (uint32_t)(4 * lane + u);
                    s_k = k - above;
                }
                above += c[u];
            }
        }
        __syncthreads();
    }
    const uint32_t thr = s_prefix;                   // the kr-th largest key; `need` of the keys equal to it are taken
    const int need = s_k;
    // ---- emit in ascending block order
    int written = 0, eq_seen = 0;
    for (int base = 0; base < nblk; base += SEL_THREADS) {
        const int j = base + tid;
        const bool in = j < nblk;
        const bool forced = in && (j < f_init || j >= f_lo);
        const bool lv = in && !forced;
        const uint32_t key = in ? pk[j] : 0u;
        int eq_tot, sel_tot;
        const int eq_rank = eq_seen + wg_prefix_count(lv && key == thr, wave_tot, tid, eq_tot);
        const bool sel = forced || (lv && key > thr) || (lv && key == thr && eq_rank < need);
        const int pos = written + wg_prefix_count(sel, wave_tot, tid, sel_tot);
        if (sel) out[pos] = j;
        written += sel_tot;
        eq_seen += eq_tot;
    }
    for (int j = written + tid; j < a.tk.topk_total; j += SEL_THREADS) out[j] = -1;
}

// ------------------------------------------------------------------------------------------ attend + merge
constexpr int AW = 8;              // waves (= selected blocks) per attend workgroup

// Up to NWV waves of a workgroup attend to one block each (j < 0: none) for the newest token of (sequence b, KV head
// h); the partial results are merged in LDS and written as partial `slot` of the pair.  Every thread of the
// workgroup calls this (barriers inside); waves past NWV only help with the final sum.  smem: NWV tiles of 16 KB.
template <int NWV>
__device__ inline void attend_partial(const DecArgs &a, int pair, int L, int slot, int j, uint16_t *smem, float (*wm)[16],
                                      float (*wl)[16]) {
    // (L = ctx[b] comes from the caller: read again here, after the caller's stores, it would be a second trip to memory
    // in front of the K/V loads)
    const int b = pair / a.hkv, h = pair - b * a.hkv;
    const int t = L - 1, bt = t / kBlock;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int m16 = lane & 15, g = lane >> 4;
    const uint16_t *kb = a.k + (int64_t)b * a.kv_batch_stride + (int64_t)h * a.kv_head_stride;
    const uint16_t *vb = a.v + (int64_t)b * a.kv_batch_stride + (int64_t)h * a.kv_head_stride;
    const float c = a.scale * LOG2E;
    TokState st;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) st.o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    st.m = -INFINITY;
    st.l = 0.f;
    if (w < NWV && j >= 0) {
        uint16_t *vtile = smem + w * TILE_ELEMS;
#pragma unroll
        for (int qi = 0; qi < 16; ++qi) load_piece(vb, a.kv_tok_stride, j, L, vtile, qi, lane);
        // K fragments as MFMA A operands, straight from global memory: row 16*kt + m16, dims 32*s + 8*g ..
        bf16x8 kf[4][4];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            const int tok = min(j * kBlock + 16 * kt + m16, L - 1);
            const uint16_t *kr = kb + (int64_t)tok * a.kv_tok_stride + g * 8;
#pragma unroll
            for (int s = 0; s < 4; ++s) kf[kt][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(kr + s * 32));
        }
        const uint16_t *qp = a.q + ((int64_t)b * a.hq + h * G + m16) * D + g * 8;
#pragma unroll
        for (int s = 0; s < 4; ++s) st.qf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(qp + s * 32));
        // every load of the wave is in flight before the first product (left alone, the scheduler requests the
        // last third of the K fragments one at a time between the products: a chain of trips to memory)
        __builtin_amdgcn_sched_barrier(0);
        const LaneOffs lo = lane_offsets(lane);
        f32x4 acc[4];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            acc[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s)
                acc[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kt][s], st.qf[s], acc[kt], 0, 0, 0);
        }
        __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);          // this wave's V tile has landed in LDS
        asm volatile("" ::: "memory");
        softmax_pv(st, acc, vtile, lo, lane, j == bt, t - j * kBlock, c);
        st.l += __shfl_xor(st.l, 16);
        st.l += __shfl_xor(st.l, 32);
    }
    if (w < NWV && g == 0) { wm[w][m16] = st.m; wl[w][m16] = st.l; }
    __syncthreads();                                  // every wave is done with its V tile: reuse as scratch
    // Each wave scales its partial to the workgroup's reference of its lane's head and lays it down as it sits in
    // registers (slot dt * 64 + lane holds dims 16 dt + 4 (lane / 16) .. + 3 of head lane % 16); the threads then
    // add the NWV partials slot by slot: 16-byte LDS traffic only, no exponentials in the sum.
    if (w < NWV) {
        float mm = wm[0][m16];
#pragma unroll
        for (int k = 1; k < NWV; ++k) mm = fmaxf(mm, wm[k][m16]);
        const float wgt = st.m == -INFINITY ? 0.f : fast_exp2((st.m - mm) * c);
        float4 *scr4 = reinterpret_cast<float4 *>(smem);           // [NWV waves][512 slots]
#pragma unroll
        for (int dt = 0; dt < 8; ++dt)
            scr4[w * (OPART / 4) + dt * 64 + lane] = make_float4(st.o[dt][0] * wgt, st.o[dt][1] * wgt, st.o[dt][2] * wgt, st.o[dt][3] * wgt);
    }
    __syncthreads();
    {
        const float4 *scr4 = reinterpret_cast<const float4 *>(smem);
        float4 *dst = reinterpret_cast<float4 *>(a.opart + ((int64_t)pair * a.nslot + slot) * OPART);
        for (int i = tid; i < OPART / 4; i += (int)blockDim.x) {
            float4 acc = scr4[i];
#pragma unroll
            for (int k = 1; k < NWV; ++k) {
                const float4 x = scr4[k * (OPART / 4) + i];
                acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
            }
            dst[i] = acc;
        }
    }
    if (tid < 16) {
        float mm = -INFINITY;
        for (int k = 0; k < NWV; ++k) mm = fmaxf(mm, wm[k][tid]);
        float ll = 0.f;
        for (int k = 0; k < NWV; ++k)
            if (wm[k][tid] != -INFINITY) ll += wl[k][tid] * fast_exp2((wm[k][tid] - mm) * c);
        float *ml = a.mlpart + ((int64_t)pair * a.nslot + slot) * 32;
        ml[tid * 2] = mm;
        ml[tid * 2 + 1] = ll;
    }
}

__global__ void __launch_bounds__(AW * 64) dec_attn_kernel(DecArgs a) {
    extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];     // AW V tiles of 16 KB, one per wave
    __shared__ float wm[AW][16], wl[AW][16];
    const int split = blockIdx.x, pair = blockIdx.y;
    const int b = pair / a.hkv;
    const int L = a.ctx[b];
    const int bt = (L - 1) / kBlock;
    const int e = split * AW + (int)(threadIdx.x >> 6);                    // entry of the block list
    int j = -1;
    if (L < a.tk.dense_below) j = e <= bt ? e : -1;
    else if (e < a.tk.topk_total) j = a.idx[(int64_t)pair * a.tk.topk_total + e];
    if (j > bt) j = -1;
    attend_partial<AW>(a, pair, L, split, j, smem, wm, wl);
}

// =========================================================================================== three-stage form
// The four kernels above are a chain of two memory bursts (compressed keys, then selected K/V blocks) separated by a
// selection that one workgroup per pair works through alone.  For the exact normalisation (lse_mode 0) the same
// step runs as
//   front  : grid (key chunks + forced splits, pairs)  the scores workgroups of above, and beside them -- independent
//            data, same launch -- workgroups that already attend to the blocks Eq. 2 keeps whatever the scores say
//            (initial and local blocks: known from the context length alone), two blocks per workgroup
//   pool   : grid (64-block groups, pairs)   every workgroup merges the pair's chunk partials into the normaliser
//            (a few KB, redundantly), normalises and group-sums its own keys, max-pools them to its 64 blocks
//   attend : grid (splits, pairs)  every workgroup first selects (radix select over the pair's <= a few thousand
//            pooled keys: no trip through memory between selection and attention), then attends to its eight
//            blocks of the top-k list
//   merge  : as above, over forced + top-k partials.
// The serial selection kernel is gone from the chain; what it did is spread over many workgroups (pool) or repeated
// by each of the few workgroups that need the result (attend).
constexpr int FW = 2;                       // forced blocks per front workgroup (2 V tiles = the 32 KB of LDS every
                                            // workgroup of that launch gets, scores workgroups included)
constexpr int PB = 64;                      // blocks per pool workgroup
constexpr int kPoolKeysMax = 2048;          // compressed keys a pool workgroup may have to hold (pool_stride * 64 + pool_len)

__global__ void __launch_bounds__(256, 4) dec_front_kernel(DecArgs a) {
    extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];     // FW V tiles of 16 KB
    __shared__ float wm[FW][16], wl[FW][16];
    const int pair = blockIdx.y;
    if ((int)blockIdx.x < a.nchunk) {
        score_chunk(a, blockIdx.x, pair);
        return;
    }
    const int f = (int)blockIdx.x - a.nchunk;             // forced split
    const int L = a.ctx[pair / a.hkv];
    const Forced fo(a.tk, L);
    const int e = f * FW + (int)(threadIdx.x >> 6);
    // (dense sequences attend to every block in the attend kernel; their forced slots stay empty)
    const int j = (L >= a.tk.dense_below && (int)(threadIdx.x >> 6) < FW && e < fo.n_forced) ? fo.forced_block(e) : -1;
    attend_partial<FW>(a, pair, L, f, j, smem, wm, wl);
}

__global__ void __launch_bounds__(256) dec_pool_kernel(DecArgs a) {
    __shared__ float red[16][16][2];
    __shared__ float lse2[16];
    __shared__ float sh[kPoolKeysMax];
    const int pair = blockIdx.y;
    const int L = a.ctx[pair / a.hkv];
    if (L < a.tk.dense_below) return;
    const Forced fo(a.tk, L);
    if (fo.kr == fo.n_rest) return;                       // everything is kept: no scores needed
    const int j0 = (int)blockIdx.x * PB;
    if (j0 >= fo.nblk) return;
    const int j1 = min(j0 + PB, fo.nblk);
    const int tid = threadIdx.x;
    const int v = visible_cmp(L - 1, a.tk.lc, a.tk.sc);
    // keys this workgroup pools: the union of its blocks' windows, clipped to the visible keys
    const int k0 = max(a.tk.pool_stride * j0 - a.tk.pool_pad, 0);
    const int k1 = min(a.tk.pool_stride * (j1 - 1) - a.tk.pool_pad + a.tk.pool_len, v);
    // their logits are requested first, so that the trip overlaps the merge of the normaliser
    constexpr int KPT = kPoolKeysMax / 256;
    const float *zb = a.z + (int64_t)pair * a.zs * G;
    float4 zr[2][4];                                      // the first two keys of this thread, 16 heads each
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int i = min(k0 + tid + u * 256, max(v - 1, 0));
        const float4 *zk = reinterpret_cast<const float4 *>(zb + (int64_t)i * G);
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) zr[u][q4] = zk[q4];
    }
    {   // log2 of sum_i 2^z per head from the chunk partials: 16 thread groups per head, then 16 -> 1
        const int head = tid & 15, pg = tid >> 4;
        const float *pp = a.part + (int64_t)pair * a.nchunk * 32 + head * 2;
        // the first 64 chunks' partials (contexts up to 131072 tokens) are requested at once, beside the logits above:
        // one trip to memory (a loop that loads as it goes makes one trip per iteration)
        constexpr int PQ = 4;
        float2 pq[PQ];
#pragma unroll
        for (int q = 0; q < PQ; ++q) pq[q] = *reinterpret_cast<const float2 *>(pp + min(pg + 16 * q, a.nchunk - 1) * 32);
        float mm = -INFINITY, ll = 0.f;
#pragma unroll
        for (int q = 0; q < PQ; ++q)
            if (pg + 16 * q < a.nchunk) mm = fmaxf(mm, pq[q].x);
        {
            const float ms = mm == -INFINITY ? 0.f : mm;
#pragma unroll
            for (int q = 0; q < PQ; ++q)
                if (pg + 16 * q < a.nchunk) ll += pq[q].y * fast_exp2(pq[q].x - ms);
        }
        for (int ch = pg + 16 * PQ; ch < a.nchunk; ch += 16) {
            const float mo = pp[ch * 32], lo = pp[ch * 32 + 1];
            const float mn = fmaxf(mm, mo);
            const float ms = mn == -INFINITY ? 0.f : mn;
            ll = ll * fast_exp2(mm - ms) + lo * fast_exp2(mo - ms);
            mm = mn;
        }
        red[pg][head][0] = mm;
        red[pg][head][1] = ll;
        __syncthreads();
        if (tid < 16) {
            float m2 = -INFINITY;
            for (int k = 0; k < 16; ++k) m2 = fmaxf(m2, red[k][tid][0]);
            float l2 = 0.f;
            for (int k = 0; k < 16; ++k)
                if (red[k][tid][0] != -INFINITY) l2 += red[k][tid][1] * fast_exp2(red[k][tid][0] - m2);
            lse2[tid] = l2 > 0.f ? m2 + __log2f(l2) : INFINITY;
        }
        __syncthreads();
    }
    // S^shared[i] = sum over the 16 heads of 2^(z[g][i] - lse2[g]) for this workgroup's keys
    float nl[G];
#pragma unroll
    for (int gq = 0; gq < G; ++gq) nl[gq] = lse2[gq];
#pragma unroll
    for (int u = 0; u < KPT; ++u) {
        const int i = k0 + tid + u * 256;
        if (i < k1) {
            float4 z4[4];
            if (u < 2) {
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) z4[q4] = zr[u][q4];
            } else {
                const float4 *zk = reinterpret_cast<const float4 *>(zb + (int64_t)i * G);
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) z4[q4] = zk[q4];
            }
            float sum = 0.f;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                sum += (fast_exp2(z4[q4].x - nl[4 * q4]) + fast_exp2(z4[q4].y - nl[4 * q4 + 1])) +
                       (fast_exp2(z4[q4].z - nl[4 * q4 + 2]) + fast_exp2(z4[q4].w - nl[4 * q4 + 3]));
            sh[i - k0] = sum;
        }
    }
    __syncthreads();
    // pooled key of every block of the group (0 for forced blocks: they take no part in the top-k)
    if (tid < j1 - j0) {
        const int j = j0 + tid;
        float m = 0.f;
        if (!fo.is_forced(j)) {
            const int lo = a.tk.pool_stride * j - a.tk.pool_pad;
            for (int u = 0; u < a.tk.pool_len; ++u) {
                const int i = lo + u;
                if (i >= 0 && i < v) m = fmaxf(m, sh[i - k0]);
            }
        }
        a.pk[(int64_t)pair * a.pk_cap + j] = __float_as_uint(m);
    }
}

// exclusive prefix count of `flag` over the workgroup's threads in thread order (+ total); two barriers
template <int NWAVES>
__device__ inline int wg_prefix_count_n(bool flag, int *wave_tot, int tid, int &total) {
    const int lane = tid & 63, w = tid >> 6;
    const uint64_t b = __ballot(flag);
    const int within = __popcll(b & ((1ull << lane) - 1ull));
    __syncthreads();                                   // previous readers of wave_tot are done
    if (lane == 0) wave_tot[w] = __popcll(b);
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int k = 0; k < NWAVES; ++k) {
        const int t = wave_tot[k];
        before += k < w ? t : 0;
        tot += t;
    }
    total = tot;
    return before + within;
}

constexpr int kSelMax = 1024;               // top-k entries (topk_total <= 1024)
constexpr int kPkLds = 4096;                // pooled keys a workgroup keeps in registers (contexts up to 262144 tokens;
                                            // longer rows are re-read from memory by every pass)

// NW waves (= blocks) per workgroup: 8 when the launch has at most one workgroup per CU anyway, 4 when it has more
// (64 KB of V tiles instead of 128: two workgroups share a CU and one's selection overlaps the other's loads).
template <int NW>
__global__ void __launch_bounds__(NW * 64) dec_attn2_kernel(DecArgs a) {
    extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];     // NW V tiles of 16 KB, one per wave
    __shared__ float wm[NW][16], wl[NW][16];
    __shared__ int wave_tot[NW];
    __shared__ uint32_t s_prefix;
    __shared__ int s_k;
    // the selection's state lives in the V tiles' memory: it is dead before the first tile is requested
    int *sel = reinterpret_cast<int *>(smem);                // [kSelMax] the top-k blocks (without the forced ones), ascending
    int(*hist)[256] = reinterpret_cast<int(*)[256]>(sel + kSelMax);     // [4][256]
    static_assert((kSelMax + 4 * 256) * 4 <= NW * TILE_ELEMS * 2, "selection state must fit in the V tiles");
    constexpr int NT = NW * 64;
    const int split = blockIdx.x, pair = blockIdx.y;
    const int b = pair / a.hkv;
    const int L = a.ctx[b];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const Forced fo(a.tk, L);
    const bool dense = L < a.tk.dense_below;
    int32_t *out = a.idx != nullptr ? a.idx + (int64_t)pair * a.tk.topk_total : nullptr;
    int j = -1;
    const int e = w < a.bpw ? split * a.bpw + w : 1 << 30;       // (waves past bpw attend to nothing)
    if (dense) {
        j = e <= fo.bt ? e : -1;
        if (out != nullptr && split == 0)
            for (int i = tid; i < a.tk.topk_total; i += NT) out[i] = -1;
    } else if (fo.kr == fo.n_rest) {
        // everything up to the query's block is kept: the blocks between the initial and the local ones
        j = e < fo.kr ? fo.f_init + e : -1;
        if (out != nullptr && split == 0)
            for (int i = tid; i < a.tk.topk_total; i += NT) out[i] = i < fo.nblk ? i : -1;
    } else {
        if (split * a.bpw >= fo.kr && !(out != nullptr && split == 0)) {
            j = -1;                                        // nothing for this workgroup: an empty partial
        } else if (fo.nblk <= kPkLds) {
            // ---- radix select (4 x 8 bits) of the kr-th largest pooled key among the live blocks; selection rule
            // and tie order as in the prefill: keys above it, then the first `need` keys equal to it by block number.
            // A thread keeps `per` consecutive blocks' keys in registers (one trip to memory, no copy in LDS); every
            // wave reduces the histogram of a pass by itself (data-parallel scan, no LDS round trips), so a pass costs
            // one barrier.
            constexpr int KPT = kPkLds / NT;
            const uint32_t *pk = a.pk + (int64_t)pair * a.pk_cap;
            const int per = (fo.nblk + NT - 1) / NT, jb0 = tid * per;
            uint32_t kreg[KPT];
            uint32_t live = 0u;                              // bit u: block jb0 + u exists and takes part in the top-k
#pragma unroll
            for (int u = 0; u < KPT; ++u) {
                const int jb = jb0 + u;
                const bool lv = u < per && jb < fo.nblk && !fo.is_forced(jb);
                kreg[u] = lv ? pk[jb] : 0u;
                live |= lv ? 1u << u : 0u;
            }
            for (int i = tid; i < 4 * 256; i += NT) (&hist[0][0])[i] = 0;
            __syncthreads();
            uint32_t prefix = 0u;
            int k = fo.kr;
            for (int pass = 3; pass >= 0; --pass) {
                const int hi_shift = 8 * (pass + 1);
#pragma unroll
                for (int u = 0; u < KPT; ++u)
                    if (((live >> u) & 1u) && (pass == 3 || (kreg[u] >> hi_shift) == prefix))
                        atomicAdd(&hist[pass][(kreg[u] >> (8 * pass)) & 255u], 1);
                __syncthreads();
                // lane l owns digits 255 - 4l .. 252 - 4l, largest first; above = number of keys with a larger digit
                int c[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) c[u] = hist[pass][255 - 4 * lane - u];
                const int mine = c[0] + c[1] + c[2] + c[3];
                int above = wave_inclusive_sum(mine) - mine;
                int digit = 0, knew = 0;
                bool found = false;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (above < k && k <= above + c[u]) {
                        found = true;
                        digit = 255 - 4 * lane - u;
                        knew = k - above;
                    }
                    above += c[u];
                }
                const int src = max(__ffsll((long long)__ballot(found)) - 1, 0);     // exactly one lane (kr >= 1 keys exist)
                prefix = (prefix << 8) | (uint32_t)__builtin_amdgcn_readlane(digit, src);
                k = __builtin_amdgcn_readlane(knew, src);
            }
            const uint32_t thr = prefix;                     // the kr-th largest key; `need` of the keys equal to it are taken
            const int need = k;
            // emission in ascending block order: one prefix count over the threads for (keys above, keys equal)
            int ca = 0, cb = 0;
#pragma unroll
            for (int u = 0; u < KPT; ++u) {
                const bool lv = ((live >> u) & 1u) != 0u;
                ca += lv && kreg[u] > thr ? 1 : 0;
                cb += lv && kreg[u] == thr ? 1 : 0;
            }
            const int packed = ca | (cb << 16);
            const int incl = wave_inclusive_sum(packed);
            if (lane == 63) wave_tot[w] = incl;
            __syncthreads();
            int before = incl - packed;
#pragma unroll
            for (int q = 0; q < NW; ++q) before += q < w ? wave_tot[q] : 0;
            int eq_before = before >> 16;
            int pos = (before & 0xffff) + min(eq_before, need);
#pragma unroll
            for (int u = 0; u < KPT; ++u) {
                if (!((live >> u) & 1u)) continue;
                bool take = kreg[u] > thr;
                if (kreg[u] == thr) {
                    take = eq_before < need;
                    ++eq_before;
                }
                if (take) sel[pos++] = jb0 + u;
            }
            __syncthreads();
            j = e < fo.kr ? sel[e] : -1;
            if (out != nullptr && split == 0) {
                // the whole list, ascending: initial blocks, the top-k, the local blocks, then -1
                const int n_loc = fo.n_forced - fo.f_init;
                for (int i = tid; i < a.tk.topk_total; i += NT) {
                    int val = -1;
                    if (i < fo.f_init) val = i;
                    else if (i < fo.f_init + fo.kr) val = sel[i - fo.f_init];
                    else if (i < fo.f_init + fo.kr + n_loc) val = fo.forced_block(i - fo.kr);
                    out[i] = val;
                }
            }
            __syncthreads();                             // the V tiles may overwrite the selection's state now
        } else {
            // the same for rows too long for the registers: every pass re-reads the pooled keys from memory
            const uint32_t *pk = a.pk + (int64_t)pair * a.pk_cap;
            for (int i = tid; i < 4 * 256; i += NT) (&hist[0][0])[i] = 0;
            if (tid == 0) { s_prefix = 0u; s_k = fo.kr; }
            __syncthreads();
            for (int pass = 3; pass >= 0; --pass) {
                const uint32_t prefix = s_prefix;
                const int hi_shift = 8 * (pass + 1);
                for (int jb = tid; jb < fo.nblk; jb += NT) {
                    if (fo.is_forced(jb)) continue;
                    const uint32_t key = pk[jb];
                    if (pass == 3 || (key >> hi_shift) == prefix) atomicAdd(&hist[pass][(key >> (8 * pass)) & 255u], 1);
                }
                __syncthreads();
                if (w == 0) {
                    // lane l owns digits 4l .. 4l+3; above = number of keys with a larger digit
                    const int k = s_k;
                    int c[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) c[u] = hist[pass][4 * lane + u];
                    const int mine = c[0] + c[1] + c[2] + c[3];
                    int run = mine;                          // inclusive suffix sum over lanes
#pragma unroll
                    for (int o = 1; o < 64; o <<= 1) {
                        const int other = __shfl_down(run, o);
                        if (lane + o < 64) run += other;
                    }
                    int above = run - mine;
#pragma unroll
                    for (int u = 3; u >= 0; --u) {
                        if (above < k && k <= above + c[u]) {
                            s_prefix = (prefix << 8) | (uint32_t)(4 * lane + u);
                            s_k = k - above;
                        }
                        above += c[u];
                    }
                }
                __syncthreads();
            }
            const uint32_t thr = s_prefix;               // the kr-th largest key; `need` of the keys equal to it are taken
            const int need = s_k;
            int written = 0, eq_seen = 0;
            for (int base = 0; base < fo.nblk; base += NT) {
                const int jb = base + tid;
                const bool lv = jb < fo.nblk && !fo.is_forced(jb);
                const uint32_t key = lv ? pk[jb] : 0u;
                int eq_tot, sel_tot;
                const int eq_rank = eq_seen + wg_prefix_count_n<NW>(lv && key == thr, wave_tot, tid, eq_tot);
                const bool take = lv && (key > thr || (key == thr && eq_rank < need));
                const int pos = written + wg_prefix_count_n<NW>(take, wave_tot, tid, sel_tot);
                if (take) sel[pos] = jb;
                written += sel_tot;
                eq_seen += eq_tot;
            }
            __syncthreads();
            j = e < fo.kr ? sel[e] : -1;
            if (out != nullptr && split == 0) {
                const int n_loc = fo.n_forced - fo.f_init;
                for (int i = tid; i < a.tk.topk_total; i += NT) {
                    int val = -1;
                    if (i < fo.f_init) val = i;
                    else if (i < fo.f_init + fo.kr) val = sel[i - fo.f_init];
                    else if (i < fo.f_init + fo.kr + n_loc) val = fo.forced_block(i - fo.kr);
                    out[i] = val;
                }
            }
            __syncthreads();                             // the V tiles may overwrite the selection's state now
        }
    }
    if (j > fo.bt) j = -1;
    attend_partial<NW>(a, pair, L, a.fsplit + split, j, smem, wm, wl);
}

// ------------------------------------------------------------------------------------------ merge
// Thread (head, group of 4 dims) combines the splits' partial results by itself, sixteen splits at a time with all of
// their loads issued before the first use: no LDS, no barrier, one round trip to memory for up to 16 splits.
constexpr int kMergeThreads = 512;
__global__ void __launch_bounds__(kMergeThreads) dec_merge_kernel(DecArgs a) {
    constexpr int R = 16;                              // splits per round
    const int pair = blockIdx.x;
    const int b = pair / a.hkv, h = pair - b * a.hkv;
    const int tid = threadIdx.x;
    const int head = tid & 15, dq = tid >> 4;          // 16 heads x 32 groups of 4 dims
    const float c = a.scale * LOG2E;
    const float *ml = a.mlpart + (int64_t)pair * a.nslot * 32 + head * 2;
    // dims 4 dq .. + 3 of this head are one 16-byte slot of a partial (see DecArgs::opart)
    const float4 *opb = reinterpret_cast<const float4 *>(a.opart + (int64_t)pair * a.nslot * OPART) +
                        (dq >> 2) * 64 + (dq & 3) * 16 + head;
    float mm = -INFINITY, ll = 0.f, o[4] = {0.f, 0.f, 0.f, 0.f};
    for (int s0 = 0; s0 < a.nslot; s0 += R) {
        float ms[R], ls[R];
        float4 ov[R];
#pragma unroll
        for (int u = 0; u < R; ++u) {
            const int s = min(s0 + u, a.nslot - 1);        // past the end: re-read the last split, weight 0 below
            const float2 m2 = *reinterpret_cast<const float2 *>(ml + s * 32);
            ms[u] = m2.x;
            ls[u] = m2.y;
            ov[u] = opb[(int64_t)s * (OPART / 4)];
        }
        // (every load above is requested before anything below is evaluated: with a branch in between the compiler
        // requests the partial outputs only after the maxima have arrived -- two trips to memory instead of one)
        __builtin_amdgcn_sched_barrier(0);
        float cm = mm;
#pragma unroll
        for (int u = 0; u < R; ++u)
            if (s0 + u < a.nslot) cm = fmaxf(cm, ms[u]);
        const float cs = cm == -INFINITY ? 0.f : cm;        // nothing attended to so far: every weight below is 0
        const float resc = mm == -INFINITY ? 0.f : fast_exp2((mm - cs) * c);
        ll *= resc;
#pragma unroll
        for (int e2 = 0; e2 < 4; ++e2) o[e2] *= resc;
#pragma unroll
        for (int u = 0; u < R; ++u) {
            const float wg = s0 + u < a.nslot && ms[u] != -INFINITY ? fast_exp2((ms[u] - cs) * c) : 0.f;
            ll += ls[u] * wg;
            o[0] += ov[u].x * wg;
            o[1] += ov[u].y * wg;
            o[2] += ov[u].z * wg;
            o[3] += ov[u].w * wg;
        }
        mm = cm;
    }
    const float inv = ll > 0.f ? 1.f / ll : 0.f;
    uint2 pk;
    pk.x = (uint32_t)float_to_bf16(o[0] * inv) | ((uint32_t)float_to_bf16(o[1] * inv) << 16);
    pk.y = (uint32_t)float_to_bf16(o[2] * inv) | ((uint32_t)float_to_bf16(o[3] * inv) << 16);
    *reinterpret_cast<uint2 *>(a.out + ((int64_t)b * a.hq + h * G + head) * D + dq * 4) = pk;
    if (a.lse != nullptr && dq == 0) a.lse[(int64_t)b * a.hq + h * G + head] = mm * a.scale + __logf(ll);
}

inline size_t align_up(size_t x, size_t al) { return (x + al - 1) / al * al; }

struct DecLayout {
    int zs, nchunk, nsplit;
    size_t off_part, off_idx, off_opart, off_ml, total;
    // three-stage form
    bool staged;
    int aw;                     // waves per attend workgroup
    int bpw;                    // blocks per attend workgroup (<= aw)
    int fsplit, nslot, pk_cap;
    size_t off_pk;
};

// the three-stage form covers the exact normalisation and pooling windows whose keys fit a pool workgroup
bool staged_params(const infllmv2_params *p) {
    return p->lse_mode == 0 && (int64_t)p->pool_stride * PB + p->pool_len <= kPoolKeysMax;
}

DecLayout dec_layout(const infllmv2_params *p, int batch, int max_ctx, int dense_blocks) {
    DecLayout d;
    const size_t pairs = (size_t)batch * p->num_kv_heads;
    const int max_nc = num_cmp(max_ctx, p->cmp_len, p->cmp_stride);
    d.zs = (int)align_up((size_t)max_nc + 4, 4);
    d.nchunk = (max_nc + CK - 1) / CK;
    if (d.nchunk < 1) d.nchunk = 1;
    d.staged = staged_params(p);
    // entries of the attend launch: the whole list (forced blocks too) in the four-kernel form, the top-k part in
    // the three-stage form; a dense sequence attends to all its blocks there either way
    const int listed = d.staged ? p->topk_total - p->n_init - p->n_local : p->topk_total;
    const int entries = listed > dense_blocks ? listed : dense_blocks;
    // three-stage form: four blocks per workgroup once eight would give more than one workgroup per CU
    d.aw = d.staged && pairs * (size_t)((entries + AW - 1) / AW) > 256 ? AW / 2 : AW;
    d.nsplit = (entries + d.aw - 1) / d.aw;
    if (d.nsplit < 1) d.nsplit = 1;
    d.bpw = d.aw;
    if (d.staged && d.aw == AW) {
        // one workgroup per CU at most: as many splits as fill the 256 CUs, each with fewer blocks (C4: 32 pairs x 8
        // splits of 7 blocks instead of 7 splits of 8 -- every CU then pulls 7/8 of the bytes)
        const int fit = (int)(256 / (pairs ? pairs : 1));
        const int ns = fit < entries ? fit : entries;
        if (ns > d.nsplit && ns <= 16 - ((p->n_init + p->n_local + FW - 1) / FW)) {
            d.nsplit = ns;
            d.bpw = (entries + ns - 1) / ns;
        }
    }
    d.fsplit = d.staged ? (p->n_init + p->n_local + FW - 1) / FW : 0;
    d.nslot = d.fsplit + d.nsplit;
    d.pk_cap = (int)align_up((size_t)(max_ctx + kBlock - 1) / kBlock + 4, 4);
    size_t off = align_up(pairs * G * d.zs * sizeof(float), 256);
    d.off_part = off;
    off += align_up(pairs * d.nchunk * 32 * sizeof(float), 256);
    d.off_idx = off;
    off += align_up(pairs * p->topk_total * sizeof(int32_t), 256);
    d.off_pk = off;
    off += d.staged ? align_up(pairs * d.pk_cap * sizeof(uint32_t), 256) : 0;
    d.off_opart = off;
    off += align_up(pairs * d.nslot * OPART * sizeof(float), 256);
    d.off_ml = off;
    off += align_up(pairs * d.nslot * 32 * sizeof(float), 256);
    d.total = off;
    return d;
}

}  // namespace

bool decode_mfma_supported(const infllmv2_params *p) {
    return p->dtype == INFLLMV2_BF16 && p->head_dim == D && p->num_q_heads / p->num_kv_heads == G;
}

// worst case over the dense fallback: a sequence just below the threshold attends to all its blocks
size_t decode_mfma_workspace(const infllmv2_params *p, int batch, int max_ctx) {
    const int dense_tokens = p->dense_threshold > 0 ? (p->dense_threshold - 1 < max_ctx ? p->dense_threshold - 1 : max_ctx) : 0;
    return dec_layout(p, batch, max_ctx, (dense_tokens + kBlock - 1) / kBlock).total;
}

int launch_decode_mfma(const infllmv2_params *p, const void *q, const void *k, const void *v, int64_t kv_batch_stride,
                       int64_t kv_head_stride, int64_t kv_tok_stride, const float *kc, int64_t kc_head_stride,
                       const int32_t *ctx_h, const int32_t *ctx_d, int batch, int32_t *idx_out, void *out, float *lse,
                       void *ws, hipStream_t stream) {
    int max_ctx = 0, dense_blocks = 0;
    for (int b = 0; b < batch; ++b) {
        if (ctx_h[b] > max_ctx) max_ctx = ctx_h[b];
        if (ctx_h[b] < p->dense_threshold) {
            const int nb = (ctx_h[b] + kBlock - 1) / kBlock;
            if (nb > dense_blocks) dense_blocks = nb;
        }
    }
    const DecLayout d = dec_layout(p, batch, max_ctx, dense_blocks);
    const int pairs = batch * p->num_kv_heads;
    DecArgs a;
    a.q = (const uint16_t *)q;
    a.k = (const uint16_t *)k;
    a.v = (const uint16_t *)v;
    a.kc = kc;
    a.ctx = ctx_d;
    a.batch = batch;
    a.hkv = p->num_kv_heads;
    a.hq = p->num_q_heads;
    a.kv_batch_stride = kv_batch_stride;
    a.kv_head_stride = kv_head_stride;
    a.kv_tok_stride = kv_tok_stride;
    a.kc_head_stride = kc_head_stride;
    a.scale = p->softmax_scale;
    a.tk = TopkArgs{p->cmp_len, p->cmp_stride, p->pool_len, p->pool_stride, p->pool_pad, p->n_init, p->n_local,
                    p->topk_total, p->dense_threshold};
    char *base = (char *)ws;
    a.z = (float *)base;
    a.part = (float *)(base + d.off_part);
    a.idx = idx_out ? idx_out : (int32_t *)(base + d.off_idx);
    a.opart = (float *)(base + d.off_opart);
    a.mlpart = (float *)(base + d.off_ml);
    a.out = (uint16_t *)out;
    a.lse = lse;
    a.zs = d.zs;
    a.nchunk = d.nchunk;
    a.nsplit = d.nsplit;
    a.lse_mode = p->lse_mode;
    a.pk = (uint32_t *)(base + d.off_pk);
    a.pk_cap = d.pk_cap;
    a.fsplit = d.fsplit;
    a.nslot = d.nslot;
    a.bpw = d.bpw;
    const size_t attn_lds = (size_t)AW * TILE_ELEMS * sizeof(uint16_t);
    if (d.staged) {
        // Larger-than-default dynamic LDS has to be enabled per kernel; the same fixed limit is set on every call,
        // so nothing has to be remembered between calls.
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(dec_attn2_kernel<AW>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)attn_lds) != hipSuccess ||
            hipFuncSetAttribute(reinterpret_cast<const void *>(dec_attn2_kernel<AW / 2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)attn_lds / 2) != hipSuccess)
            return INFLLMV2_ERR_HIP;
        a.idx = idx_out;                     // written by the attend kernel only when the caller wants the list
        const int groups = ((max_ctx + kBlock - 1) / kBlock + PB - 1) / PB;
        hipLaunchKernelGGL(dec_front_kernel, dim3(d.nchunk + d.fsplit, pairs), dim3(256),
                           (size_t)FW * TILE_ELEMS * sizeof(uint16_t), stream, a);
        hipLaunchKernelGGL(dec_pool_kernel, dim3(groups, pairs), dim3(256), 0, stream, a);
        if (d.aw == AW)
            hipLaunchKernelGGL(dec_attn2_kernel<AW>, dim3(d.nsplit, pairs), dim3(AW * 64), attn_lds, stream, a);
        else
            hipLaunchKernelGGL(dec_attn2_kernel<AW / 2>, dim3(d.nsplit, pairs), dim3(AW * 32), attn_lds / 2, stream, a);
        hipLaunchKernelGGL(dec_merge_kernel, dim3(pairs), dim3(kMergeThreads), 0, stream, a);
        return hip_status(hipGetLastError());
    }

    // group sum + max-pool + top-k run as one workgroup per pair with the score row in LDS
    const int sh_cap = (d.zs + 3) / 4 * 4;
    // (one pooled key per selection block: however many compressed keys a block spans)
    const size_t sel_lds = ((size_t)sh_cap + (size_t)(max_ctx + kBlock - 1) / kBlock + 4) * sizeof(float);
    if (sel_lds > kSelLdsMax) return INFLLMV2_ERR_UNSUPPORTED;     // before anything is launched
    // Larger-than-default dynamic LDS has to be enabled per kernel; the same fixed limits are set on every call, so
    // nothing has to be remembered between calls.
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(dec_select_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSelLdsMax) != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void *>(dec_attn_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)attn_lds) != hipSuccess)
        return INFLLMV2_ERR_HIP;
    hipLaunchKernelGGL(dec_scores_kernel, dim3(d.nchunk, pairs), dim3(256), 0, stream, a);
    hipLaunchKernelGGL(dec_select_kernel, dim3(pairs), dim3(SEL_THREADS), sel_lds, stream, a, sh_cap);
    hipLaunchKernelGGL(dec_attn_kernel, dim3(d.nsplit, pairs), dim3(AW * 64), attn_lds, stream, a);
    hipLaunchKernelGGL(dec_merge_kernel, dim3(pairs), dim3(kMergeThreads), 0, stream, a);
    return hip_status(hipGetLastError());
}

}  // namespace ifv2
