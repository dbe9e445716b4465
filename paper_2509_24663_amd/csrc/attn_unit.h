// Building blocks of the prefill tile kernel and the decode attention kernel: asynchronous global -> LDS copies,
// LDS tile layouts and the (token, block) MFMA units.  bf16 data, G = 16 heads per KV head, d_h = 128.
// Two units live here.  The decode unit (first part of the file) works on the caches as they are: K fragments
// come straight from global memory, V through a row-major LDS tile read with transposing loads.  The prefill unit
// (second part) works on a K tile and a pre-transposed V^T tile and is arranged around the issue-port and LDS
// bandwidth limits described there.
#pragma once
#include "common.h"

namespace ifv2 {
namespace attn_unit {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void glb_void;

constexpr int D = 128;            // head dim
constexpr int G = 16;             // heads per KV head
constexpr int TILE_ELEMS = kBlock * D;            // one K or V block in LDS: 64 rows x 256 B, unpadded
constexpr int STAGE_ELEMS = 2 * TILE_ELEMS;       // K then V: 32 KB per stage
constexpr float LOG2E = 1.4426950408889634f;
constexpr int WAIT_VMCNT0 = 0x0F70;               // s_waitcnt vmcnt(0), other counters untouched
constexpr int WAIT_LGKMCNT0 = 0xC07F;             // s_waitcnt lgkmcnt(0), other counters untouched

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// 16 bytes per lane, global -> LDS without passing through registers: lane l's data lands at dst + 16 l (dst is
// wave-uniform).  Issued as assembly on purpose: the compiler then does not know that LDS is written behind its
// back and does not stall later LDS reads of *other* tiles on the vector-memory counter.  Every reader of the
// destination must be ordered by an explicit s_waitcnt vmcnt + barrier, which the callers do.
__device__ inline void async_copy16(const void *src, const uint16_t *dst) {
    const uint32_t lds = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void *)dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds), "v"(src) : "memory", "m0");
}

// The same with a wave-uniform 64-bit base (held in scalar registers) plus a 32-bit byte offset per lane, so that
// a loop can step the base with scalar arithmetic only.  lds is the LDS byte address of the destination.
__device__ inline void async_copy16(const void *sbase, uint32_t voff, uint32_t lds) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(sbase) : "memory", "m0");
}

__device__ inline uint32_t lds_address(const void *p) { return (uint32_t)(uintptr_t)(lds_void *)p; }

// =====================================================================================================
// Decode unit
//
// One 1 KB piece (4 rows) of a K or V block: global -> LDS, asynchronously.  Lane l fills LDS slot
// (row 4*q16 + l/16, physical chunk l%16), which holds logical 16-byte chunk (l%16) ^ (row%16) of that row.
// Rows past the end of the sequence re-read the last valid row (finite data, always masked by causality).
__device__ inline void load_piece(const uint16_t *base, int64_t tok_stride, int j, int len, uint16_t *tile, int q16,
                                  int lane) {
    const int row = 4 * q16 + (lane >> 4);
    const int chunk = (lane & 15) ^ (row & 15);
    const int tok = min(j * kBlock + row, len - 1);
    const uint16_t *src = base + (int64_t)tok * tok_stride + chunk * 8;
    async_copy16(src, tile + q16 * 512);
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

__device__ inline LaneOffs lane_offsets(int lane) {
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

// ---- S^T = K_blk Q_t^T with the K block in a swizzled LDS tile: acc[kt][r] = key 16*kt + 4*(lane/16) + r.
// The 16 operand reads go through a rolling window of 8 registers sets, and consecutive MFMAs write
// different accumulators, so LDS latency and MFMA latency overlap instead of adding up.
__device__ inline void qk_from_lds(f32x4 (&acc)[4], const bf16x8 (&qf)[4], const uint16_t *ktile, const LaneOffs &lo) {
    bf16x8 f[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)      // i -> (s = i / 4, kt = i % 4)
        f[i] = *reinterpret_cast<const bf16x8 *>(ktile + (i & 3) * 16 * D + lo.kx[i >> 2]);
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) acc[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int kt = i & 3, s = i >> 2;
        acc[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[i & 7], qf[s], acc[kt], 0, 0, 0);
        if (i + 8 < 16) f[i & 7] = *reinterpret_cast<const bf16x8 *>(ktile + kt * 16 * D + lo.kx[s + 2]);
    }
}

// max over the four 16-lane rows of a wave (lanes with equal lane % 16), without going through LDS
__device__ inline float rows_max(float x) {
    const unsigned u = __float_as_uint(x);
    const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    const float m1 = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const unsigned v = __float_as_uint(m1);
    const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

// The running reference st.m of the online softmax need not be the exact row maximum: any value shared by the
// lanes of a head works as long as 2^(c (z - m)) stays far from overflow.  It is therefore only refreshed
// (cross-lane max, rescale of O and l) when some logit exceeds it by more than this many powers of two.
constexpr float kMaxSlack = 8.0f;

// ---- online softmax over the 64 logits of a block and O^T += V_blk^T P^T (V block in a swizzled LDS tile)
__device__ inline void softmax_pv(TokState &st, f32x4 (&acc)[4], const uint16_t *vt, const LaneOffs &lo, int lane,
                                  bool diag, int key_limit, float c) {
    const int g = lane >> 4;
    if (__builtin_amdgcn_readfirstlane(diag)) {       // only the query's own block needs the causal mask
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (16 * kt + 4 * g + r > key_limit) acc[kt][r] = -INFINITY;
    }
    float mx = fmaxf(fmaxf(acc[0][0], acc[0][1]), fmaxf(acc[0][2], acc[0][3]));
#pragma unroll
    for (int kt = 1; kt < 4; ++kt) mx = fmaxf(mx, fmaxf(fmaxf(acc[kt][0], acc[kt][1]), fmaxf(acc[kt][2], acc[kt][3])));
    if (__any(mx * c > st.m * c + kMaxSlack)) {
        const float m_new = fmaxf(st.m, rows_max(mx));
        const float alpha = fast_exp2((st.m - m_new) * c);
        st.m = m_new;
        st.l *= alpha;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) st.o[dt] *= alpha;
    }
    const float nmc = -st.m * c;
    float ls = 0.f;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            acc[kt][r] = fast_exp2(__builtin_fmaf(acc[kt][r], c, nmc));
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
    // 16 MFMAs, i -> (s2 = i / 8, dt = i % 8): consecutive ones write different accumulators; the V^T
    // operands (two transposing reads each) go through a rolling window of 8
    typedef __attribute__((address_space(3))) short4v lds_s4;
    short4v v0[8], v1[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        v0[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4 *)(vt + lo.vx[i]));
        v1[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4 *)(vt + 16 * D + lo.vx[i]));
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int dt = i & 7, s2 = i >> 3;
        const short8v v8 = __builtin_shufflevector(v0[dt], v1[dt], 0, 1, 2, 3, 4, 5, 6, 7);
        st.o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v8), pb[s2], st.o[dt], 0, 0, 0);
        if (i < 8) {
            v0[dt] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4 *)(vt + 32 * D + lo.vx[dt]));
            v1[dt] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4 *)(vt + 48 * D + lo.vx[dt]));
        }
    }
}

// =====================================================================================================
// Prefill unit: one K/V block (both tiles in one LDS stage) against the token held by this wave.
//
// The vector unit and the matrix core share one issue port per SIMD (4 clocks per instruction, an MFMA keeps
// the matrix core busy for 16), so every vector instruction in the unit costs matrix-core time unless fewer
// than three of them accompany each MFMA.  The softmax is therefore arranged so that nothing is computed that
// the MFMA can produce for free:
//   * Q is multiplied by softmax_scale * log2(e) once, when it is loaded, and
//   * the accumulator of S^T = K Q^T is seeded with minus the running reference of the online softmax,
// so the MFMA result is already the exponent of 2 and a logit costs one v_exp, one add (row sum) and half a
// pack instruction.  The reference is lazy: any value shared by the lanes of a head works as long as the
// exponents stay far from overflow, so it only moves when the probabilities show that an exponent was large.
//
// LDS bandwidth is the other limit (a one-token unit reads 32 KB for 32 MFMAs), and 8-byte transposing reads run
// at half the rate of 16-byte reads.  V therefore comes from a transposed copy (V^T, one [128 dims][64 keys]
// tile per block, made by a small pre-pass), so that both operands are fetched with ds_read_b128:
//   * K tile  [64 keys][128 dims], 256-byte rows, 16-byte chunk c of row r stored at chunk c ^ f(r),
//     f(r) = 4 * ((r >> 3) & 3) + (r & 3);
//   * V^T tile [128 dims][64 keys], 128-byte rows, chunk c of row r stored at chunk c ^ ((r >> 1) & 7): two rows
//     span the 64 banks, so the 16 lanes of a group (rows m .. m + 15, same logical chunk) must differ in
//     (r & 1, position) -- a swizzle by r & 7 would send rows r and r + 8 to the same banks.
// Row m of the A operand of S^T's key tile kt is key 32 (kt / 2) + 8 (m / 4) + 4 (kt % 2) + (m % 4): with that
// order the exponents a lane ends up with are exactly the eight consecutive keys 32 s2 + 8 (lane / 16) .. + 7 it
// must supply as B operand of PV k-step s2, and f(key) = m for every kt, so one address per k-step serves all
// key tiles through the instruction's immediate offset.
constexpr int VT_TILE_ELEMS = D * kBlock;            // one V^T block: 128 rows x 128 B

struct LaneOffs2 {
    int kx[4];         // K operand, k-step s: element offset of (row 8 (m16 / 4) + m16 % 4, logical chunk 4s + g)
    int vx[2];         // V^T operand, k-step s2: element offset of (row m16, logical chunk 4 s2 + g)
};

__device__ inline LaneOffs2 lane_offsets2(int lane) {
    LaneOffs2 o;
    const int m16 = lane & 15, g = lane >> 4;
    const int krow = 8 * (m16 >> 2) + (m16 & 3);
#pragma unroll
    for (int s = 0; s < 4; ++s) o.kx[s] = krow * D + (((4 * s + g) ^ m16) << 3);
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) o.vx[s2] = m16 * kBlock + (((4 * s2 + g) ^ ((m16 >> 1) & 7)) << 3);
    return o;
}

// Per-lane byte offsets of the asynchronous loads that fill the two tiles; piece q is 1 KB of LDS.
// K piece q (rows 4q .. 4q+3 of the block): lane l fills (row 4q + l / 16, physical chunk l % 16).
__device__ inline void k_piece_src(int q, int lane, int &row, int &chunk) {
    row = 4 * q + (lane >> 4);
    chunk = (lane & 15) ^ (4 * ((row >> 3) & 3) + (row & 3));
}
// V^T piece q (rows 8q .. 8q+7 of the tile): lane l fills (row 8q + l / 8, physical chunk l % 8).
__device__ inline uint32_t vt_piece_src_bytes(int q, int lane) {
    const int row = 8 * q + (lane >> 3);
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    return (uint32_t)(row * kBlock + chunk * 8) * 2u;
}

struct Tok {
    bf16x8 qf[4];      // Q_t * softmax_scale * log2(e) as MFMA B operand: head = lane % 16, dims ks*32 + (lane/16)*8 ..
    f32x4 o[8];        // O_t^T: dim tile dt, dims dt*16 + 4*(lane/16) + r, head = lane % 16
    f32x4 nm;          // minus the reference (log2 units) in all four slots: seed of the S^T accumulator
    float l;           // this lane's share of the running sum
    bool fresh;        // no block consumed yet (wave-uniform)
};

// a lane's 16 probabilities may sum to this much before the reference moves (each is then < 2^12)
constexpr float kSumSlack = 4096.0f;

__device__ inline void tok_init(Tok &t) {
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) t.o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    t.nm = f32x4{0.f, 0.f, 0.f, 0.f};
    t.l = 0.f;
    t.fresh = true;
}

// Q fragment scaled by c and rounded to bf16 (round to nearest even)
__device__ inline bf16x8 scale_q(uint4 raw, float c) {
    const bf16x8 q = __builtin_bit_cast(bf16x8, raw);
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (__bf16)((float)q[i] * c);
    return r;
}

__device__ inline bf16x8 k_frag(const uint16_t *ktile, const LaneOffs2 &lo, int i) {     // i -> (s = i / 4, kt = i % 4)
    const int kt = i & 3;
    return *reinterpret_cast<const bf16x8 *>(ktile + (32 * (kt >> 1) + 4 * (kt & 1)) * D + lo.kx[i >> 2]);
}
__device__ inline bf16x8 v_frag(const uint16_t *vtile, const LaneOffs2 &lo, int i) {     // i -> (s2 = i / 8, dt = i % 8)
    return *reinterpret_cast<const bf16x8 *>(vtile + (i & 7) * 16 * kBlock + lo.vx[i >> 3]);
}

// 2^exponent for the 16 exponents of a lane, packed as the B operand of the two PV k-steps (slot i = key
// 32 s2 + 8g + i); returns their sum
__device__ inline float probs(const f32x4 (&acc)[4], bf16x8 (&pb)[2]) {
    float ls = 0.f;
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float p0 = fast_exp2(acc[2 * s2][r]), p1 = fast_exp2(acc[2 * s2 + 1][r]);
            ls += p0 + p1;
            pb[s2][r] = (__bf16)p0;
            pb[s2][4 + r] = (__bf16)p1;
        }
    return ls;
}

// Exponents of one token -> probabilities, with the causal mask of the token's own block and the lazy reference.
// The probabilities are computed with the reference as it is; only if a lane's sum of them says that an exponent
// was large (or this is the token's first block) is the reference moved and the work redone from the exponents,
// which are still in acc.  The common case then has no maximum to compute at all.
template <bool OWN>
__device__ inline void softmax_tok(Tok &t, f32x4 (&acc)[4], bf16x8 (&pb)[2], int g, int key_limit) {
    if (OWN) {
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (32 * (kt >> 1) + 8 * g + 4 * (kt & 1) + r > key_limit) acc[kt][r] = -INFINITY;
    }
    float ls = probs(acc, pb);
    if (t.fresh || __any(!(ls < kSumSlack))) {
        float mx = fmaxf(fmaxf(acc[0][0], acc[0][1]), acc[0][2]);
        mx = fmaxf(fmaxf(mx, acc[0][3]), acc[1][0]);
        mx = fmaxf(fmaxf(mx, acc[1][1]), acc[1][2]);
        mx = fmaxf(fmaxf(mx, acc[1][3]), acc[2][0]);
        mx = fmaxf(fmaxf(mx, acc[2][1]), acc[2][2]);
        mx = fmaxf(fmaxf(mx, acc[2][3]), acc[3][0]);
        mx = fmaxf(fmaxf(mx, acc[3][1]), acc[3][2]);
        mx = fmaxf(mx, acc[3][3]);
        // move the reference of every head to its current maximum (never down once there is history)
        float delta = rows_max(mx);
        float alpha = 1.0f;
        if (!t.fresh) {
            delta = fmaxf(delta, 0.f);
            alpha = fast_exp2(-delta);
        }
        t.fresh = false;
#pragma unroll
        for (int kt = 0; kt < 4; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[kt][r] -= delta;
#pragma unroll
        for (int r = 0; r < 4; ++r) t.nm[r] -= delta;
        t.l *= alpha;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) t.o[dt] *= alpha;
        ls = probs(acc, pb);
    }
    t.l += ls;
}

// One token against one block.  OWN: the block is the token's own and keys past key_limit are masked.
template <bool OWN>
__device__ inline void unit(Tok &t, const uint16_t *stage, const LaneOffs2 &lo, int lane, int key_limit) {
    const uint16_t *ktile = stage, *vtile = stage + TILE_ELEMS;
    constexpr int W = 4;               // operand fetches run W MFMAs ahead
    f32x4 acc[4];
    bf16x8 pb[2];
    bf16x8 f[W];
    // ---- exponents: S^T seeded with minus the reference
#pragma unroll
    for (int i = 0; i < W; ++i) f[i] = k_frag(ktile, lo, i);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int kt = i & 3, s = i >> 2;
        acc[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[i % W], t.qf[s], s == 0 ? t.nm : acc[kt], 0, 0, 0);
        if (i + W < 16) f[i % W] = k_frag(ktile, lo, i + W);
    }
    // V^T fragments of the first k-step are requested before the softmax so that they arrive under it
#pragma unroll
    for (int i = 0; i < W; ++i) f[i] = v_frag(vtile, lo, i);
    softmax_tok<OWN>(t, acc, pb, lane >> 4, key_limit);
    // ---- O^T += V^T P^T
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int dt = i & 7, s2 = i >> 3;
        t.o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[i % W], pb[s2], t.o[dt], 0, 0, 0);
        if (i + W < 16) f[i % W] = v_frag(vtile, lo, i + W);
    }
}

}  // namespace attn_unit
}  // namespace ifv2
