// Stage 4 on the matrix cores: block-sparse causal attention (Appendix Alg. 2) and dense causal attention
// (Eq. 1 / Appendix Alg. 3) for bf16 data with G = 16 query heads per KV head and d_h = 128.
//
// Alg. 2 gives every token a private pass over its selected K/V blocks.  Here a workgroup owns a tile of
// T consecutive tokens of one KV head instead: it forms the union of the tile's block lists, brings each
// K/V block of the union into LDS once, and every token that selected the block consumes it from there.
// Neighbouring tokens share blocks (all init/local blocks, and whichever top-k blocks they agree on), so the
// gather traffic from L2 / HBM drops by the sharing factor while the arithmetic stays exactly the
// per-token softmax attention of Alg. 2.
//
// Data movement: a small pre-pass writes V^T, one [128 dims][64 keys] tile per block (zero-padded past the end
// of a sequence), into the caller's workspace.  K blocks and V^T tiles then go from global memory straight
// into LDS (global_load_lds, 16 bytes per lane, no register staging) with the 16-byte chunks of a row
// XOR-swizzled so that the 16-byte operand reads below are spread over all banks.
//
// Per (token, block) the 16 heads of the group are one MFMA tile side.  S^T = K_blk Q_t^T is 4 key tiles x
// 4 k-steps of v_mfma_f32_16x16x32_bf16 (A = K rows from LDS, B = Q_t held in registers), so a lane owns
// one head and 16 keys: the online softmax needs two cross-lane steps when its reference moves and none for
// the row sum (kept as per-lane partial sums until the end).  The key rows are assigned to the MFMA rows in
// a permuted order that makes the probabilities of a lane exactly the B operand of O^T += V_blk^T P^T
// (8 dim tiles x 2 k-steps), whose A operand comes from the V^T tile.  Dense attention is the same kernel
// with "every block, every token".
//
// Schedule: the waves of a tile walk the union in lock step, one barrier per interval of two entries (dense: two
// consecutive blocks), the next interval's blocks landing in the other half of a four-stage LDS buffer meanwhile.
//
// Compile-time switches exist for timing experiments only (a build with either gives wrong results; they are
// never defined in the library build): ATTN_TIMING_NO_LOADS leaves out the global -> LDS copies (every stage holds the
// sequence's first block instead: real data, so the softmax takes its usual path and the operands toggle as usual), and
// ATTN_TIMING_NO_BARRIER the barrier that ends an interval.  What the kernel's time is made of is measured with them.
// A third one, ATTN_TIMING_CLOCK, keeps the outputs correct but writes, instead of lse, where each wave's time in the
// main loop went (constant 100 MHz clock: issuing copies, units, waiting for its own copies, waiting at the barrier).
// ATTN_TIMING_NEAR=N takes every copy from the sequence's first N blocks (are the copies bound by where they come from?).
// ATTN_TIMING_DROP_PRIVATE=C leaves the union entries with at most C consumers out of the walk (what do they cost?).
#include <type_traits>

#include "attn_unit.h"

namespace ifv2 {

namespace {

using namespace attn_unit;

struct AttnArgs {
    const uint16_t *q, *k, *v;
    const uint16_t *vt;      // V^T blocks: [kv head][block of the batch][128 dims][64 keys]
    int nblk_total;          // blocks of the whole batch (sum over sequences of ceil(len / 64))
    const int32_t *idx;
    uint16_t *out;
    float *lse;
    RowMap map;
    int hq, topk_total, dense_below;
    float scale;
    int nb_cap;        // words reserved in LDS for the per-block token masks
    int list_cap;      // entries reserved for the union list
};

// NW waves with one token each, SLOTS union entries per barrier interval.
template <int NW, int SLOTS>
struct TileKernel {
    static constexpr int T = NW;
    static constexpr int NTHR = NW * 64;
    static constexpr int NSTAGE = 2 * SLOTS;        // double buffering of an interval's blocks
    static constexpr int PPW = 32 / NW;             // one-KB load pieces per wave and block
    static constexpr int NONE = 0xffff;            // no block (block numbers are kept in 16 bits)
    static_assert(32 % NW == 0, "32 one-KB load instructions are dealt round-robin to the waves");
    static_assert(SLOTS == 1 || SLOTS == 2, "one or two entries per interval");

    // which of the CU's four SIMDs this wave runs on (hardware id register, bits 5:4)
    __device__ static inline int simd_id() { return (int)__builtin_amdgcn_s_getreg(4 | (4 << 6) | (1 << 11)); }

    // An interval holds two consecutive entries of the union list, and between its barriers a SIMD works through
    // the units of the waves it hosts, so an interval lasts about as long as its busiest SIMD.  The list (all of
    // it but the tile's own block, which stays last) is therefore re-paired: each wave takes a contiguous, even
    // sized range of entries and repeatedly joins its first remaining entry to the one that raises the pair's
    // busiest SIMD the least.  Partners stay a few entries apart, so the walk remains nearly ascending
    // (neighbouring tiles then touch the same blocks at about the same time, which the L2 likes).
    __device__ static inline void pair_entries(int2 *rec, int body, int w, int lane, const uint32_t *simd_waves) {
        const int pairs = body / 2;
        const int lo = 2 * (pairs * w / NW), hi = 2 * (pairs * (w + 1) / NW);
        const int n = hi - lo;
        if (n < 4 || n > 64) return;                        // nothing to choose / more entries than lanes: left as is
        bool live = lane < n;
        const int2 r = live ? rec[lo + lane] : make_int2(NONE, 0);
        uint32_t loads = 0u;                                // consumers per SIMD, one byte each
#pragma unroll
        for (int sd = 0; sd < 4; ++sd) loads |= (uint32_t)__popc((uint32_t)r.y & simd_waves[sd]) << (8 * sd);
        auto max_byte = [](uint32_t x) -> int {
            return (int)max(max(x & 0xffu, (x >> 8) & 0xffu), max((x >> 16) & 0xffu, x >> 24));
        };
        const int own_max = max_byte(loads);
        for (int pos = lo; pos < hi; pos += 2) {
            // first: the live entry with the smallest block number, which keeps the walk close to ascending
            const int first = __ffsll((long long)__ballot(live)) - 1;
            const uint32_t lf = (uint32_t)__builtin_amdgcn_readlane((int)loads, first);
            if (lane == first) { rec[pos] = r; live = false; }
            // second: the live entry whose company costs the least beyond what it would cost alone
            const int extra = max_byte(lf + loads) - own_max;
            int second = 0;
            for (int c = 0; c <= NW / 4; ++c) {
                const uint64_t b = __ballot(live && extra == c);
                if (b) { second = __ffsll((long long)b) - 1; break; }
            }
            if (lane == second) { rec[pos + 1] = r; live = false; }
        }
    }

    __device__ static void run(const AttnArgs &a, int num_tiles) {
        extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
        uint16_t *stages = smem;
        uint32_t *masks = reinterpret_cast<uint32_t *>(smem + NSTAGE * STAGE_ELEMS);
        int2 *rec = reinterpret_cast<int2 *>(masks + a.nb_cap);          // union list: (block, token mask) per entry
        __shared__ int s_seq, s_tile, s_blk0, s_ne, s_ni;
        __shared__ uint32_t s_simd_waves[4];                             // waves (= tokens) resident on each SIMD
#ifdef ATTN_TIMING_CLOCK
        __shared__ uint32_t s_busy_ticks[2][NW];                         // per interval parity: each wave's ticks from the
                                                                         // barrier to its arrival at the next one
#endif

        const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
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
            int rem = tile_id, s = 0, blk0 = 0;
            for (; s < a.map.batch; ++s) {
                const int ln = a.map.cu[s + 1] - a.map.cu[s];
                const int nt = (ln + T - 1) / T;
                if (rem < nt) break;
                rem -= nt;
                blk0 += (ln + kBlock - 1) / kBlock;
            }
            s_seq = s;
            s_tile = rem;
            s_blk0 = blk0;
            for (int i = 0; i < 4; ++i) s_simd_waves[i] = 0u;
        }
        __syncthreads();
        if (SLOTS == 2 && lane == 0) atomicOr(&s_simd_waves[simd_id()], 1u << w);     // read after later barriers
        const int seq = __builtin_amdgcn_readfirstlane(s_seq);
        if (seq >= a.map.batch) return;
        const int tok0 = a.map.cu[seq], len = a.map.cu[seq + 1] - tok0;
        const int t0 = __builtin_amdgcn_readfirstlane(s_tile) * T;       // first token of the tile (position in the sequence)
        const int ntok = min(T, len - t0);
        const int bt = t0 / kBlock, nblk = bt + 1;       // T divides 64: the tile lies in one block
        const bool dense = a.idx == nullptr || len < a.dense_below;
        const int row0 = tok0 + t0;                      // packed row of the tile's first token
        const uint16_t *kb = a.k + (int64_t)tok0 * a.map.kv_tok_stride + (int64_t)h * a.map.kv_head_stride;
        const uint16_t *vtb = a.vt + ((int64_t)h * a.nblk_total + __builtin_amdgcn_readfirstlane(s_blk0)) * VT_TILE_ELEMS;
        const uint32_t full = ntok >= 32 ? 0xffffffffu : ((1u << ntok) - 1u);

        // ---- union of the tile's block lists: masks[j] has bit ti set if token ti selected block j.  The tile's
        // own block is the largest one any of its tokens selects, and every token selects it: it is the last entry.
        int ni;                                          // number of barrier intervals
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
                    uint32_t mk = j < nblk ? masks[j] : 0u;
#ifdef ATTN_TIMING_DROP_PRIVATE
                    // timing experiment only (results are wrong): entries with at most this many consumers are left out
                    if (j != bt && __popc(mk) <= ATTN_TIMING_DROP_PRIVATE) mk = 0u;
#endif
                    const uint64_t b = __ballot(mk != 0u);
                    if (mk != 0u) rec[base + __popcll(b & ((1ull << lane) - 1ull))] = make_int2(j, (int)mk);
                    base += __popcll(b);
                }
                if (lane == 0) { s_ne = base; s_ni = SLOTS == 2 && base > 0 ? base / 2 + 1 : base; }
            }
            __syncthreads();
            ni = __builtin_amdgcn_readfirstlane(s_ni);
            if (SLOTS == 2) {
                pair_entries(rec, __builtin_amdgcn_readfirstlane(s_ne) - 1, w, lane, s_simd_waves);
                __syncthreads();
            }
        } else {
            ni = SLOTS == 2 ? nblk / 2 + 1 : nblk;     // pairs of blocks, the tile's own block alone at the end
        }
        // Interval i -> its blocks and consumer masks (unused slot: block NONE, mask 0).  With SLOTS == 2 an
        // interval covers two consecutive entries of the union, so that a SIMD usually has two or more units to
        // overlap between one pair of barriers; the tile's own block (the last entry) is alone in the last interval.
        const int ne = dense ? nblk : __builtin_amdgcn_readfirstlane(s_ne);
        // (packed into two words -- block numbers and consumer masks in 16 bits each -- because the record of the next
        // interval waits in vector registers while a unit runs)
        auto pack = [](int j0, int mk0, int j1, int mk1) -> int2 {
            return make_int2((j0 & 0xffff) | (j1 << 16), (mk0 & 0xffff) | (mk1 << 16));
        };
        if (!dense && SLOTS == 2) {
            // the list becomes the list of packed interval records, in place (one thread per interval: ni <= NTHR
            // because the list has at most T * topk_total + 1 <= 2 * NTHR entries, which the host checks), so that the
            // main loop fetches a record with one LDS read and nothing to compute on it
            int2 r0 = make_int2(NONE, 0), r1 = make_int2(NONE, 0);
            if (tid < ni) {
                if (tid == ni - 1) {
                    r0 = rec[ne - 1];
                } else {
                    r0 = rec[2 * tid];
                    if (2 * tid + 1 < ne - 1) r1 = rec[2 * tid + 1];
                }
            }
            __syncthreads();
            if (tid < ni) rec[tid] = pack(r0.x, r0.y, r1.x, r1.y);
            __syncthreads();
        }
        auto interval = [&](int i) -> int2 {
            if (dense) {
                if (SLOTS == 1) return pack(i, (int)full, NONE, 0);
                if (i == ni - 1) return pack(ne - 1, (int)full, NONE, 0);
                const int j1 = 2 * i + 1 < ne - 1 ? 2 * i + 1 : NONE;
                return pack(2 * i, (int)full, j1, j1 != NONE ? (int)full : 0);
            }
            if (SLOTS == 1) {
                const int2 r = rec[i];
                return pack(r.x, r.y, NONE, 0);
            }
            return rec[i];
        };

        // ---- loads: a block is 32 one-KB pieces (16 of the K tile: 4 rows each; 16 of the V^T tile: 8 rows each); wave w
        // copies K piece w and V^T piece w of every block.  A piece's source is a wave-uniform base (sequence, head,
        // block, piece: scalar arithmetic) plus a per-lane byte offset that never changes, except that the sequence's
        // last, partial K block re-reads its last valid row (finite data, always masked by causality); that block can
        // only be the tile's own, which is alone in the last interval.  The V^T copy is zero-padded instead.
        //
        // A wave's instructions issue in order, so whatever a wave with a unit in the current interval spends on the
        // next interval's copies -- address arithmetic included -- delays that unit, and the interval lasts as long as
        // its slowest wave: the code below is the shortest there is for four copies (every piece offset folded into
        // per-wave constants, 32-bit block stride, the partial block handled by the last interval's own function).
        static_assert(NW == 16, "wave w copies piece w of the 16 pieces of a tile");
        constexpr uint32_t kTileBytes = TILE_ELEMS * 2, kStageBytes = STAGE_ELEMS * 2;
        const uint32_t blk_bytes = (uint32_t)a.map.kv_tok_stride * (uint32_t)(kBlock * sizeof(uint16_t));   // < 2^31: the stride is < 2^24
        const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(stages));
        const int own_rows = len - bt * kBlock;          // rows of the tile's own block that exist (1..64 counts)
        uint32_t off_k_w, off_v_w;
        {
            int row, chunk;
            k_piece_src(w, lane, row, chunk);
            off_k_w = (uint32_t)((row - 4 * w) * (int)a.map.kv_tok_stride + chunk * 8) * 2u;
            off_v_w = vt_piece_src_bytes(w, lane) - (uint32_t)w * 1024u;
        }
        const char *kb_w = reinterpret_cast<const char *>(kb) + (uint64_t)w * (blk_bytes / 16u);
        const char *vtb_w = reinterpret_cast<const char *>(vtb) + (uint32_t)w * 1024u;
        const uint32_t lds_w = lds0 + (uint32_t)w * 1024u;
#ifdef ATTN_TIMING_NO_LOADS
        bool timing_fill = false;
#endif
        // this wave's sixteenth of the interval whose blocks are jj (two 16-bit block numbers), into buffer buf
        auto issue = [&](uint32_t jj, int buf) {
#ifdef ATTN_TIMING_NO_LOADS
            if (!timing_fill) return;                   // timing experiment only (results are garbage)
#endif
            uint32_t j0 = jj & 0xffffu, j1 = jj >> 16;
            const bool two = SLOTS == 2 && j1 != (uint32_t)NONE;
#ifdef ATTN_TIMING_NEAR
            j0 %= ATTN_TIMING_NEAR;                     // timing experiment only: all copies come from a few blocks
            j1 %= ATTN_TIMING_NEAR;
#endif
            const uint32_t dst = lds_w + (uint32_t)buf * (SLOTS * kStageBytes);
            async_copy16(kb_w + (uint64_t)j0 * blk_bytes, off_k_w, dst);
            async_copy16(vtb_w + (j0 << 14), off_v_w, dst + kTileBytes);
            if (two) {
                async_copy16(kb_w + (uint64_t)j1 * blk_bytes, off_k_w, dst + kStageBytes);
                async_copy16(vtb_w + (j1 << 14), off_v_w, dst + kStageBytes + kTileBytes);
            }
        };
        // the last interval: the tile's own block alone, possibly the sequence's partial last block
        auto issue_last = [&](int buf) {
#ifdef ATTN_TIMING_NO_LOADS
            if (!timing_fill) return;
#endif
            const uint32_t dst = lds_w + (uint32_t)buf * (SLOTS * kStageBytes);
            int row, chunk;
            k_piece_src(w, lane, row, chunk);
            const uint32_t off = (uint32_t)(min(row, own_rows - 1) * (int)a.map.kv_tok_stride + chunk * 8) * 2u;
            async_copy16(reinterpret_cast<const char *>(kb) + (uint64_t)bt * blk_bytes, off, dst);
            async_copy16(vtb_w + ((uint32_t)bt << 14), off_v_w, dst + kTileBytes);
        };
        int2 r_cur = ni > 0 ? interval(0) : make_int2(0, 0);
#ifdef ATTN_TIMING_NO_LOADS
        // every stage holds the sequence's first block for the whole tile: real data (the softmax takes its usual
        // path, the matrix core sees operands that toggle as usual), but nothing is copied afterwards
        timing_fill = true;
        for (int b2 = 0; b2 < 2; ++b2) issue(0u, b2);
        timing_fill = false;
#endif
        if (ni == 1) issue_last(0);
        else if (ni > 1) issue((uint32_t)__builtin_amdgcn_readfirstlane(r_cur.x), 0);

        // ---- this wave's token
        Tok st;
        const int m16 = lane & 15, g = lane >> 4;
        const int ti = w;
        {
            float cm;
            int ce;
            split_scale(a.scale * LOG2E, cm, ce);
            const uint16_t *qp = a.q + ((int64_t)(row0 + ti) * a.hq + h * G + m16) * D + g * 8;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                uint4 raw = ti < ntok ? *reinterpret_cast<const uint4 *>(qp + s * 32) : make_uint4(0, 0, 0, 0);
                st.qf[s] = scale_q(raw, ce);
            }
            tok_init(st, __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, cm))));
        }
        const uint32_t kx = k_lane_bytes(lane), vx = v_lane_bytes(lane);

        // Main loop: while interval i is consumed from one buffer, the blocks of interval i + 1 land in the other
        // (every wave left that buffer before the barrier that ended interval i - 1).  The interval records are
        // read one iteration ahead, so their LDS latency hides behind the unit.
        int2 r_next = ni > 1 ? interval(1) : r_cur;
#ifdef ATTN_TIMING_CLOCK
        uint64_t ck_issue = 0, ck_units = 0, ck_wait = 0, ck_barrier = 0, ck_critical = 0;
        const uint64_t ck_start = wall_clock64();
#endif
        __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
        __syncthreads();
        auto step = [&](auto own, int i) {
            constexpr bool OWN = decltype(own)::value;
            const int j0 = __builtin_amdgcn_readfirstlane(r_cur.x) & 0xffff;
            const uint32_t mks = (uint32_t)__builtin_amdgcn_readfirstlane(r_cur.y);
            const uint32_t mk0 = mks & 0xffffu, mk1 = SLOTS == 2 ? mks >> 16 : 0u;
#ifdef ATTN_TIMING_CLOCK
            const uint64_t ck0 = wall_clock64();
#endif
            // A CU accepts the interval's 64 copies at ~64 bytes per clock and a wave's instructions issue in order, so
            // a wave that issued its copies first would start its unit ~0.3 us late.  Waves without a unit in this
            // interval issue at once; the others from inside their first unit, once its S^T products are out.
            const bool u0 = ((mk0 >> w) & 1u) != 0u, u1 = SLOTS == 2 && ((mk1 >> w) & 1u) != 0u;
            // 0: nothing to issue (any more); 1: the last interval; 2: any other
            int mode = i + 1 >= ni ? 0 : i + 2 == ni ? 1 : 2;
            const uint32_t jj_next = (uint32_t)__builtin_amdgcn_readfirstlane(r_next.x);
            auto issue_now = [&]() {
                if (mode == 1) issue_last((i + 1) & 1);
                if (mode == 2) issue(jj_next, (i + 1) & 1);
                mode = 0;
            };
            if (!(u0 || u1)) issue_now();
#ifdef ATTN_TIMING_CLOCK
            const uint64_t ck1 = wall_clock64();
            ck_issue += ck1 - ck0;
#endif
            r_cur = r_next;
            if (i + 2 < ni) r_next = interval(i + 2);
            const uint32_t stage = lds0 + (uint32_t)(((i & 1) * SLOTS) * STAGE_ELEMS * 2);
            // (consecutive tests rather than the arms of one branch: the compiler would otherwise merge the
            // identical operand reads of the two units above the branch and run out of registers)
            if (u0) unit<OWN>(st, stage, kx, vx, lane, t0 + w - j0 * kBlock, issue_now);
            if (u1) unit<false>(st, stage + STAGE_ELEMS * 2, kx, vx, lane, 0, issue_now);
#ifdef ATTN_TIMING_CLOCK
            const uint64_t ck2 = wall_clock64();
            ck_units += ck2 - ck1;
#endif
            __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);        // this wave's pieces of the next interval have landed
#ifdef ATTN_TIMING_CLOCK
            const uint64_t ck3 = wall_clock64();
            ck_wait += ck3 - ck2;
            if (lane == 0) s_busy_ticks[i & 1][w] = (uint32_t)(ck3 - ck0);
#endif
#ifndef ATTN_TIMING_NO_BARRIER
            __syncthreads();
#endif
#ifdef ATTN_TIMING_CLOCK
            ck_barrier += wall_clock64() - ck3;
            {   // the interval's last arrival: how long the wave that everybody waited for was under way
                uint32_t mx = 0;
                for (int k = 0; k < NW; ++k) mx = max(mx, s_busy_ticks[i & 1][k]);
                ck_critical += mx;
            }
#endif
        };
        for (int i = 0; i < ni - 1; ++i) step(std::false_type{}, i);
        if (ni > 0) step(std::true_type{}, ni - 1);

        // ---- normalise and store
        if (ti < ntok) {
            float l = st.l;
            l += __shfl_xor(l, 16);
            l += __shfl_xor(l, 32);
            const float inv = l > 0.f ? 1.0f / l : 0.f;
            uint16_t *op = a.out + ((int64_t)(row0 + ti) * a.hq + h * G + m16) * D + g * 4;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                uint2 pk;
                pk.x = (uint32_t)float_to_bf16(st.o[dt][0] * inv) | ((uint32_t)float_to_bf16(st.o[dt][1] * inv) << 16);
                pk.y = (uint32_t)float_to_bf16(st.o[dt][2] * inv) | ((uint32_t)float_to_bf16(st.o[dt][3] * inv) << 16);
                *reinterpret_cast<uint2 *>(op + dt * 16) = pk;
            }
            // log-sum-exp in natural units: the reference and the row sum are kept in powers of two
#ifdef ATTN_TIMING_CLOCK
            // timing experiment: instead of lse, heads 0-6 of the group get this wave's 100 MHz ticks spent issuing
            // copies, in units, waiting for its own copies, at the barrier, in the whole main loop, the number of
            // intervals, and the sum over intervals of the last-arriving wave's ticks from barrier to barrier
            if (a.lse != nullptr && g == 0 && m16 < 7) {
                const uint64_t vals[7] = {ck_issue, ck_units, ck_wait, ck_barrier, wall_clock64() - ck_start, (uint64_t)ni, ck_critical};
                a.lse[(int64_t)(h * G + m16) * a.map.total_rows + row0 + ti] = (float)vals[m16];
            }
#else
            if (a.lse != nullptr && g == 0)
                a.lse[(int64_t)(h * G + m16) * a.map.total_rows + row0 + ti] = (__log2f(l) - st.nr) * 0.6931471805599453f;
#endif
        }
    }
};

// V -> V^T: one workgroup per (block of the batch, KV head); keys past the end of a sequence become zeros.
__global__ void __launch_bounds__(256) vt_transpose_kernel(const uint16_t *v, uint16_t *vt, RowMap map, int nblk_total) {
    __shared__ uint16_t tile[kBlock][D + 8];
    __shared__ int s_tok, s_rows;
    const int tid = threadIdx.x, h = blockIdx.y;
    if (tid == 0) {
        int rem = blockIdx.x, s = 0;
        for (; s < map.batch; ++s) {
            const int nb = (map.cu[s + 1] - map.cu[s] + kBlock - 1) / kBlock;
            if (rem < nb) break;
            rem -= nb;
        }
        s_tok = s < map.batch ? map.cu[s] + rem * kBlock : 0;
        s_rows = s < map.batch ? min(kBlock, map.cu[s + 1] - map.cu[s] - rem * kBlock) : 0;
    }
    __syncthreads();
    const int rows = s_rows;
    const uint16_t *src = v + (int64_t)s_tok * map.kv_tok_stride + (int64_t)h * map.kv_head_stride;
    for (int i = tid; i < kBlock * (D / 8); i += 256) {
        const int r = i / (D / 8), c = i % (D / 8);
        uint4 x = make_uint4(0, 0, 0, 0);
        if (r < rows) x = *reinterpret_cast<const uint4 *>(src + (int64_t)r * map.kv_tok_stride + c * 8);
        *reinterpret_cast<uint4 *>(&tile[r][c * 8]) = x;
    }
    __syncthreads();
    uint16_t *dst = vt + ((int64_t)h * nblk_total + blockIdx.x) * VT_TILE_ELEMS;
    for (int i = tid; i < D * (kBlock / 8); i += 256) {
        const int d = i / (kBlock / 8), c = i % (kBlock / 8);
        uint16_t e[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) e[u] = tile[c * 8 + u][d];
        uint4 x;
        x.x = e[0] | ((uint32_t)e[1] << 16);
        x.y = e[2] | ((uint32_t)e[3] << 16);
        x.z = e[4] | ((uint32_t)e[5] << 16);
        x.w = e[6] | ((uint32_t)e[7] << 16);
        *reinterpret_cast<uint4 *>(dst + d * kBlock + c * 8) = x;
    }
}

template <int NW, int SLOTS>
__global__ void __launch_bounds__(NW * 64) attn_tile_kernel(AttnArgs a, int num_tiles) {
    TileKernel<NW, SLOTS>::run(a, num_tiles);
}

template <int NW, int SLOTS>
int launch_tile(const Launch &L, const AttnArgs &a0, const int32_t *cu_h) {
    constexpr int T = NW;
    AttnArgs a = a0;
    int64_t tiles = 0;
    for (int s = 0; s < L.map.batch; ++s) tiles += (cu_h[s + 1] - cu_h[s] + T - 1) / T;
    if (tiles == 0) return INFLLMV2_OK;
    const int nb_max = (L.max_len + kBlock - 1) / kBlock;
    a.nb_cap = a.idx ? (nb_max + 3) / 4 * 4 : 0;
    a.list_cap = a.idx ? (min(nb_max, T * L.p->topk_total) + 1) / 2 * 2 : 0;
    // stages, block masks, union list (8 bytes per entry)
    const size_t lds = (size_t)2 * SLOTS * STAGE_ELEMS * sizeof(uint16_t) +
                       (size_t)a.nb_cap * 4 + (size_t)a.list_cap * 8;
    if (lds > 160 * 1024 - 256 || nb_max >= 0xffff) return INFLLMV2_ERR_UNSUPPORTED;     // does not fit: the caller pairs nothing
    if (SLOTS == 2 && a.list_cap / 2 + 1 > NW * 64) return INFLLMV2_ERR_UNSUPPORTED;      // one thread packs one interval record
    auto kern = attn_tile_kernel<NW, SLOTS>;
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

// the V^T copy: one [128 dims][64 keys] tile per block and KV head
size_t attn_fwd_ws_bytes(const infllmv2_params *p, const BatchTotals &t) {
    if (!attn_mfma_supported(p)) return 0;
    return align256((size_t)t.blocks * p->num_kv_heads * VT_TILE_ELEMS * sizeof(uint16_t));
}

int launch_attn_mfma(const Launch &L, const void *q, const void *k, const void *v, const int32_t *idx,
                     int dense_below, void *out, float *lse, const int32_t *cu_h) {
    // 16-byte vector loads need 8-element aligned strides
    if (L.map.kv_tok_stride % 8 != 0 || L.map.kv_head_stride % 8 != 0) return INFLLMV2_ERR_UNSUPPORTED;
    // per-lane load offsets inside one block are kept in 32 bits
    if (L.map.kv_tok_stride <= 0 || L.map.kv_tok_stride >= (1 << 24)) return INFLLMV2_ERR_UNSUPPORTED;
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
    // V^T copy for the tile kernel, in the caller's workspace
    int64_t nblk_total = 0;
    for (int s = 0; s < L.map.batch; ++s) nblk_total += (cu_h[s + 1] - cu_h[s] + kBlock - 1) / kBlock;
    if (nblk_total == 0) return INFLLMV2_OK;
    void *ws = L.ws;
    if (ws == nullptr || L.ws_bytes < (size_t)nblk_total * L.p->num_kv_heads * VT_TILE_ELEMS * sizeof(uint16_t))
        return INFLLMV2_ERR_WORKSPACE_TOO_SMALL;
    a.vt = (const uint16_t *)ws;
    a.nblk_total = (int)nblk_total;
    hipLaunchKernelGGL(vt_transpose_kernel, dim3((unsigned)nblk_total, L.p->num_kv_heads), dim3(256), 0, L.stream,
                       a.v, (uint16_t *)ws, L.map, (int)nblk_total);
    int rc = hip_status(hipGetLastError());
    if (rc == INFLLMV2_OK) {
        // Two entries per interval when the four LDS stages that needs fit next to the block masks (with block lists:
        // sequences up to about 384K tokens; dense calls keep no masks), else one.
        rc = INFLLMV2_ERR_UNSUPPORTED;
        rc = launch_tile<16, 2>(L, a, cu_h);
        if (rc == INFLLMV2_ERR_UNSUPPORTED) rc = launch_tile<16, 1>(L, a, cu_h);
    }
    return rc;
}

}  // namespace ifv2
