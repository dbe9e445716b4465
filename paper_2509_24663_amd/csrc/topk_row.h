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

// srow: the row's group scores (global or LDS), t: query position, out: topk_total entries.
// NCH > 0: pooled keys live in NCH registers per lane (blocks j = c*64 + lane, needs nblk <= 64*NCH);
// NCH == 0: they live in lk[] (LDS, at least 64*ceil(nblk/64) words owned by this wave).
template <int NCH>
__device__ inline void topk_row(const float *srow, int t, const TopkArgs &a, int32_t *out, uint32_t *lk, int lane) {
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
        float m = 0.f;
        for (int u = 0; u < a.pool_len; ++u) {
            int i = lo + u;
            if (i >= 0 && i < v) m = fmaxf(m, srow[i]);
        }
        return __float_as_uint(m);
    };
    if (NCH > 0) {
#pragma unroll
        for (int c = 0; c < NCH; ++c)
            if (c < nch) keys[c] = pooled(c * 64 + lane);
    } else {
        for (int c = 0; c < nch; ++c) lk[c * 64 + lane] = pooled(c * 64 + lane);
    }
    // a lane's slot is "live" if it is a real, non-forced block
    auto live = [&](int j) -> bool { return j < nblk && !(j < f_init || j >= f_lo); };
    auto key_at = [&](int c) -> uint32_t { return NCH > 0 ? keys[c] : lk[c * 64 + lane]; };

    // ---- k-th largest by bit descent (kr >= 0; kr == 0 keeps only the forced blocks)
    if (kr > 0) {
        uint32_t p = 0;
        bool exact = false;
        for (int b = 31; b >= 0; --b) {
            const uint32_t cand = p | (1u << b);
            int cnt = 0;
            if (NCH > 0) {
#pragma unroll
                for (int c = 0; c < NCH; ++c)
                    if (c < nch) cnt += __popcll(__ballot(live(c * 64 + lane) && keys[c] >= cand));
            } else {
                for (int c = 0; c < nch; ++c) cnt += __popcll(__ballot(live(c * 64 + lane) && key_at(c) >= cand));
            }
            if (cnt >= kr) {
                p = cand;
                if (cnt == kr) { exact = true; break; }
            }
        }
        if (exact) {
            thr_gt = p - 1;            // exactly kr keys are >= p
            need = 0;
        } else {
            // p is the kr-th largest value; more than kr keys are >= p, so some equal ones are dropped
            int gt = 0;
            if (NCH > 0) {
#pragma unroll
                for (int c = 0; c < NCH; ++c)
                    if (c < nch) gt += __popcll(__ballot(live(c * 64 + lane) && keys[c] > p));
            } else {
                for (int c = 0; c < nch; ++c) gt += __popcll(__ballot(live(c * 64 + lane) && key_at(c) > p));
            }
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
