// Selection of one (token, KV head) row by one wavefront: max-pool the group scores to one value per
// 64-token block (Sec. 3.3, Eq. 6), always keep the initial and local blocks, take the top-k of the
// remaining blocks (Sec. 3.2, Eq. 2).
//
// Scores are non-negative floats, so their bit patterns order like unsigned integers; the k-th largest
// pooled score is found by descending over the 32 bits (count of keys >= candidate via ballot + popcount),
// stopping early as soon as exactly k keys qualify.  Equal scores at the threshold are resolved towards the
// smaller block index, and the result is written in ascending block order with a ballot prefix -- no sort,
// no atomics, bitwise deterministic.
#pragma once
#include "common.h"

namespace ifv2 {

struct TopkArgs {
    int lc, sc, pool_len, pool_stride, pool_pad, n_init, n_local, topk_total;
    int dense_below;   // rows of sequences shorter than this get an all -1 list (they attend densely)
};

// Bit descent over the first N register chunks: on return p is either (exact) a value with exactly kr keys
// >= p, or the kr-th largest key, with gt = number of keys > p.
template <int N, int NK>
__device__ inline void descend(const uint32_t (&keys)[NK], int kr, uint32_t &p, bool &exact, int &gt) {
    static_assert(N <= NK, "chunk count");
    for (int b = 31; b >= 0; --b) {
        const uint32_t cand = p | (1u << b);
        int cnt = 0;
#pragma unroll
        for (int c = 0; c < N; ++c) cnt += __popcll(__ballot(keys[c] >= cand));
        if (cnt >= kr) {
            p = cand;
            if (cnt == kr) { exact = true; return; }
        }
    }
#pragma unroll
    for (int c = 0; c < N; ++c) gt += __popcll(__ballot(keys[c] > p));
}

// srow: the row's group scores (global or LDS), t: query position, out: topk_total entries.
// NCH > 0: pooled keys live in NCH registers per lane (blocks j = c*64 + lane, needs nblk <= 64*NCH);
// NCH == 0: they live in lk[] (LDS, at least 64*ceil(nblk/64) words owned by this wave).
// MODE: where the pooled scores come from.
enum : int {
    TOPK_POOL_ANY = 0,    // srow holds scores per compressed key; any pooling window
    TOPK_POOL_FAST = 1,   // the same for the paper's window (l = 5, s = 4, no shift), srow 16-byte aligned: vector loads
    TOPK_POOLED = 2,      // srow already holds one score per block (the score kernel pooled on chip); entry j is
                          // defined iff its window has a visible key, max(stride j - pad, 0) < v
};
// cand: kCandPerWave (key, block) pairs of LDS owned by this wave (used when NCH > kCandChunks).
constexpr int kCandChunks = 4, kCandPerWave = 64 * kCandChunks;
constexpr int kBoundBits = 12;          // leading key bits (below the sign) resolved on the lane maxima
template <int NCH, int MODE = TOPK_POOL_ANY>
__device__ inline void topk_row(const float *srow, int t, const TopkArgs &a, int32_t *out, uint32_t *lk, uint2 *cand,
                                int lane) {
    const int bt = t / kBlock, nblk = bt + 1;
    const int v = visible_cmp(t, a.lc, a.sc);
    const int nch = (nblk + 63) >> 6;

    // forced blocks: [0, n_init) and (bt - n_local, bt]
    const int f_init = min(a.n_init, nblk);
    const int f_lo = max(0, bt - a.n_local + 1);
    const int n_forced = f_init + (bt - f_lo + 1) - max(0, f_init - f_lo);
    const int n_rest = nblk - n_forced;
    const int kr = min(a.topk_total - a.n_init - a.n_local, n_rest);

    uint32_t thr_gt = 0xffffffffu, thr_eq = 0xffffffffu;   // select key > thr_gt, or key == thr_eq (first `need`)
    int need = 0;
    uint32_t keys[NCH > 0 ? NCH : 1];

    if (kr == n_rest) {
        // everything up to the query's block is kept: no scores needed
        for (int j = lane; j < a.topk_total; j += 64) out[j] = j < nblk ? j : -1;
        return;
    }

    // ---- pooled keys
#pragma unroll
    for (int c = 0; c < (NCH > 0 ? NCH : 1); ++c) keys[c] = 0;
    auto pooled = [&](int j) -> uint32_t {
        if (j >= nblk) return 0u;
        const bool forced = j < f_init || j >= f_lo;
        if (forced) return 0u;
        const int lo = a.pool_stride * j - a.pool_pad;
        if (MODE == TOPK_POOLED) return max(lo, 0) < v ? __float_as_uint(srow[j]) : 0u;
        float m = 0.f;
        for (int u = 0; u < a.pool_len; ++u) {
            int i = lo + u;
            if (i >= 0 && i < v) m = fmaxf(m, srow[i]);
        }
        return __float_as_uint(m);
    };
    if (NCH > 0 && MODE == TOPK_POOL_FAST) {
        // pool window = [4j, 4j+5): one aligned 16-byte load plus one scalar per block, all issued up front
        // with addresses clamped into the visible prefix (so nothing branches and nothing is read out of
        // bounds); invisible or forced entries are masked afterwards.
        const int vlast = max(v - 1, 0);
#pragma unroll
        for (int c0 = 0; c0 < NCH; c0 += 8) {
            float4 q4[8];
            float f5[8];
#pragma unroll
            for (int c = c0; c < c0 + 8 && c < NCH; ++c) {
                const int i0 = 4 * (c * 64 + lane);
                q4[c - c0] = *reinterpret_cast<const float4 *>(srow + min(i0, vlast & ~3));
                f5[c - c0] = srow[min(i0 + 4, vlast)];
            }
#pragma unroll
            for (int c = c0; c < c0 + 8 && c < NCH; ++c) {
                const int j = c * 64 + lane, i0 = 4 * j;
                float m = 0.f;
                m = i0 < v ? fmaxf(m, q4[c - c0].x) : m;
                m = i0 + 1 < v ? fmaxf(m, q4[c - c0].y) : m;
                m = i0 + 2 < v ? fmaxf(m, q4[c - c0].z) : m;
                m = i0 + 3 < v ? fmaxf(m, q4[c - c0].w) : m;
                m = i0 + 4 < v ? fmaxf(m, f5[c - c0]) : m;
                const bool dead = j >= nblk || j < f_init || j >= f_lo;
                keys[c] = dead ? 0u : __float_as_uint(m);
            }
        }
    } else if (NCH > 0 && MODE == TOPK_POOLED) {
        // all loads first, addresses clamped into the row (entry bt always exists); undefined, forced and
        // out-of-range entries are masked afterwards
        float x[NCH > 0 ? NCH : 1];
#pragma unroll
        for (int c = 0; c < NCH; ++c) x[c] = srow[min(c * 64 + lane, bt)];
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int j = c * 64 + lane;
            const bool dead = j >= nblk || j < f_init || j >= f_lo || !(max(a.pool_stride * j - a.pool_pad, 0) < v);
            keys[c] = dead ? 0u : __float_as_uint(x[c]);
        }
    } else if (NCH > 0) {
#pragma unroll
        for (int c = 0; c < NCH; ++c)
            if (c < nch) keys[c] = pooled(c * 64 + lane);
    } else {
        for (int c = 0; c < nch; ++c) lk[c * 64 + lane] = pooled(c * 64 + lane);
    }
    // a lane's slot is "live" if it is a real, non-forced block
    auto live = [&](int j) -> bool { return j < nblk && !(j < f_init || j >= f_lo); };
    auto key_at = [&](int c) -> uint32_t { return NCH > 0 ? keys[c] : lk[c * 64 + lane]; };

    // ---- long rows: shrink the problem to a few hundred candidates first.
    // Each lane's largest key is one element of the row, so the kr-th largest of the 64 lane maxima is a lower
    // bound of the kr-th largest key (kr <= 64).  Its leading bits, found by a descent over that single register,
    // give a bound L that typically leaves 100-250 keys >= L out of thousands.  Those are compacted, in
    // ascending block order, into LDS; threshold search and emission then run over at most kCandChunks
    // registers instead of NCH.  Rows where that does not work out (too many candidates, L = 0, kr > 64) take
    // the general path below.
    if (NCH > kCandChunks && kr > 0 && kr <= 64 && nch > kCandChunks) {
        uint32_t lm = 0;
#pragma unroll
        for (int c = 0; c < NCH; ++c) lm = max(lm, keys[c]);
        uint32_t L = 0;
        for (int b = 30; b > 30 - kBoundBits; --b) {
            const uint32_t c2 = L | (1u << b);
            if (__popcll(__ballot(lm >= c2)) >= kr) L = c2;
        }
        if (L != 0) {
            const uint64_t below = (1ull << lane) - 1ull;
            int total = 0;
#pragma unroll
            for (int c = 0; c < NCH; ++c) {
                const bool in = keys[c] >= L;                    // dead slots hold 0 < L
                const uint64_t bal = __ballot(in);
                const int pos = total + __popcll(bal & below);
                if (in && pos < kCandPerWave) cand[pos] = make_uint2(keys[c], (uint32_t)(c * 64 + lane));
                total += __popcll(bal);
            }
            if (total <= kCandPerWave) {
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
                __builtin_amdgcn_wave_barrier();
                uint32_t ck[kCandChunks], cj[kCandChunks];
#pragma unroll
                for (int u = 0; u < kCandChunks; ++u) {
                    const uint2 e = u * 64 + lane < total ? cand[u * 64 + lane] : make_uint2(0u, 0u);
                    ck[u] = e.x;
                    cj[u] = e.y;
                }
                // total >= kr keys are >= L, so the kr-th largest key of the row is among the candidates
                uint32_t p = 0;
                bool exact = false;
                int gt = 0;
                if (total <= 128) descend<2>(ck, kr, p, exact, gt);
                else descend<kCandChunks>(ck, kr, p, exact, gt);
                const uint32_t above = exact ? p - 1 : p;        // keys > above are in
                const int need_eq = exact ? 0 : kr - gt;         // plus the first need_eq keys == p
                // forced initial blocks, the selected candidates (ascending), forced local blocks
                for (int j = lane; j < f_init; j += 64) out[j] = j;
                int written = f_init, eq_seen = 0;
#pragma unroll
                for (int u = 0; u < kCandChunks; ++u) {
                    const bool is_eq = need_eq > 0 && ck[u] == p;   // padding holds 0 < L <= p
                    const uint64_t eqb = __ballot(is_eq);
                    const bool sel = ck[u] > above || (is_eq && eq_seen + __popcll(eqb & below) < need_eq);
                    const uint64_t sb = __ballot(sel);
                    if (sel) out[written + __popcll(sb & below)] = (int32_t)cj[u];
                    written += __popcll(sb);
                    eq_seen += __popcll(eqb);
                }
                for (int j = f_lo + lane; j <= bt; j += 64) out[written + j - f_lo] = j;
                written += bt - f_lo + 1;
                for (int j = written + lane; j < a.topk_total; j += 64) out[j] = -1;
                return;
            }
        }
    }

    // ---- k-th largest by bit descent (kr >= 0; kr == 0 keeps only the forced blocks).
    // Dead slots (forced blocks, blocks past the query) hold key 0 and every candidate is >= 1, so they are
    // never counted; the register variant therefore runs straight-line over a compile-time chunk count.
    if (kr > 0) {
        uint32_t p = 0;
        bool exact = false;
        int gt = 0;
        if (NCH > 0) {
            if (nch * 4 <= NCH) descend<(NCH + 3) / 4>(keys, kr, p, exact, gt);
            else if (nch * 2 <= NCH) descend<(NCH + 1) / 2>(keys, kr, p, exact, gt);
            else descend<(NCH > 0 ? NCH : 1)>(keys, kr, p, exact, gt);
        } else {
            for (int b = 31; b >= 0; --b) {
                const uint32_t cand = p | (1u << b);
                int cnt = 0;
                for (int c = 0; c < nch; ++c) cnt += __popcll(__ballot(key_at(c) >= cand));
                if (cnt >= kr) {
                    p = cand;
                    if (cnt == kr) { exact = true; break; }
                }
            }
            if (!exact)
                for (int c = 0; c < nch; ++c) gt += __popcll(__ballot(key_at(c) > p));
        }
        if (exact) {
            thr_gt = p - 1;            // exactly kr keys are >= p
            need = 0;
        } else {
            // p is the kr-th largest value; more than kr keys are >= p, so some equal ones are dropped
            thr_gt = p;
            thr_eq = p;
            need = kr - gt;
        }
    }

    // ---- emit in ascending block order
    int written = 0, eq_seen = 0;
    const uint64_t lt_mask = (1ull << lane) - 1ull;
    auto emit = [&](int c, uint32_t key) {
        const int j = c * 64 + lane;
        const bool forced = j < nblk && (j < f_init || j >= f_lo);
        const bool lv = live(j);
        const bool is_eq = lv && need > 0 && key == thr_eq;
        const uint64_t eqb = __ballot(is_eq);
        const int eq_rank = eq_seen + __popcll(eqb & lt_mask);
        const bool sel = forced || (lv && kr > 0 && key > thr_gt) || (is_eq && eq_rank < need);
        const uint64_t sb = __ballot(sel);
        if (sel) out[written + __popcll(sb & lt_mask)] = j;
        written += __popcll(sb);
        eq_seen += __popcll(eqb);
    };
    if (NCH > 0) {
#pragma unroll
        for (int c = 0; c < NCH; ++c)
            if (c < nch) emit(c, keys[c]);
    } else {
        for (int c = 0; c < nch; ++c) emit(c, key_at(c));
    }
    for (int j = written + lane; j < a.topk_total; j += 64) out[j] = -1;
}

}  // namespace ifv2
