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

// Operand addresses.  K operand of k-step s: row 8 (m16 / 4) + m16 % 4 (+ a constant per key tile), logical chunk
// 4s + g, stored at chunk (4s + g) ^ m16 = (g ^ m16) ^ 4s: the byte offset of k-step s is that of k-step 0 with
// bits 6-7 flipped by s, so one register per lane (plus an exclusive-or when the address is formed) serves all
// k-steps.  Likewise the V^T operand of k-step s2: row m16 (+ 16 per dim tile), chunk (4 s2 + g) ^ ((m16 >> 1) & 7).
__device__ inline uint32_t k_lane_bytes(int lane) {
    const int m16 = lane & 15, g = lane >> 4;
    return (uint32_t)((8 * (m16 >> 2) + (m16 & 3)) * D + ((g ^ m16) << 3)) * 2u;
}
__device__ inline uint32_t v_lane_bytes(int lane) {
    const int m16 = lane & 15, g = lane >> 4;
    return (uint32_t)(m16 * kBlock + ((g ^ ((m16 >> 1) & 7)) << 3)) * 2u;
}
typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8;
__device__ inline bf16x8 lds_read16(uint32_t byte_addr) { return *(lds_bf16x8 *)(uintptr_t)byte_addr; }

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
    bf16x8 qf[4];      // Q_t * 2^ce (exact) as MFMA B operand: head = lane % 16, dims ks*32 + (lane/16)*8 ..
    f32x4 o[8];        // O_t^T: dim tile dt, dims dt*16 + 4*(lane/16) + r, head = lane % 16
    float nr;          // minus the reference of the online softmax, in powers of two
    float l;           // this lane's share of the running sum
    float cm;          // mantissa of softmax_scale * log2(e): probability = 2^(cm * accumulator + nr)
    float slack;       // a lane's probabilities of a half block may sum to this much before the reference moves;
                       // negative while no block has been consumed yet, so that the first one always sets it
                       // (a value rather than a flag: a branch on a flag lets the compiler move the
                       // exponentials out from between the products)
};

// a lane's 8 probabilities of a half block may sum to this much before the reference moves (each is then < 2^12)
constexpr float kSumSlack = 4096.0f;

// softmax_scale * log2(e) = cm * 2^ce with 0.5 <= cm < 1.  The power of two goes into Q (exact in bf16), the
// mantissa multiplies the fp32 accumulator (in the same fused multiply-add that subtracts the reference), so the
// logits are those of Q as stored (Alg. 2 computes S from Q itself; rounding Q * scale back to bf16 would move
// every logit by ~1e-3).
__device__ inline void split_scale(float c, float &cm, int &ce) { cm = frexpf(c, &ce); }

__device__ inline void tok_init(Tok &t, float cm) {
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) t.o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    t.nr = 0.f;
    t.l = 0.f;
    t.cm = cm;
    t.slack = -1.0f;
}

// Q fragment times 2^ce: exact unless the result leaves bf16's exponent range
__device__ inline bf16x8 scale_q(uint4 raw, int ce) {
    const bf16x8 q = __builtin_bit_cast(bf16x8, raw);
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (__bf16)ldexpf((float)q[i], ce);
    return r;
}

// kb / vb: LDS byte address of the stage (a multiple of 1024) plus k_lane_bytes / v_lane_bytes of the lane.  The
// k-step is applied by exclusive-or after the stage address has been added (the stage address has no low bits, so
// that is the same thing) -- formed the other way round, the compiler keeps a register per k-step alive for the whole
// kernel.  Key tile / dim tile offsets are instruction immediates.
__device__ inline bf16x8 k_frag(uint32_t kb, int kt, int s) {
    return lds_read16((kb ^ (uint32_t)(64 * s)) + (uint32_t)((32 * (kt >> 1) + 4 * (kt & 1)) * D * 2));
}
__device__ inline bf16x8 v_frag(uint32_t vb, int dt, int s2) {
    return lds_read16((vb ^ (uint32_t)(64 * s2)) + (uint32_t)(TILE_ELEMS * 2 + dt * 16 * kBlock * 2));
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

__device__ inline uint32_t pack_bf16(float lo, float hi) {
    return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){lo, hi}, bf16x2));
}

// A lane's share of a half block (32 keys): the 8 exponents a0[0..3], a1[0..3] become the B operand of the PV
// k-step of that half (slot e = key 32 half + 8g + e).  exponent e -> probability; the causal mask of the token's own
// block is applied on the way and written back, so that a later move of the reference sees the masked exponents.
template <bool OWN>
__device__ inline float prob_step(f32x4 &a0, f32x4 &a1, int e, float (&p)[2], u32x4 &pb, float cm, float nr, int key0,
                                  int key_limit) {
    float x = e < 4 ? a0[e & 3] : a1[e & 3];
    if (OWN && key0 + e > key_limit) {
        x = -INFINITY;
        if (e < 4) a0[e & 3] = x; else a1[e & 3] = x;
    }
    const float q = fast_exp2(__builtin_fmaf(x, cm, nr));
    p[e & 1] = q;
    if (e & 1) {
        uint32_t w = pack_bf16(p[0], p[1]);
        asm volatile("" : "+v"(w));        // packed here, not after the branch that follows the half block
        pb[e >> 1] = w;
    }
    return q;
}

// The lazy reference.  Probabilities are computed with the reference as it is; only if a lane's sum of them says
// that an exponent was large (or this is the token's first half block) is the reference moved to the half block's
// maximum, everything accumulated so far rescaled, and the half block's probabilities redone from the exponents,
// which are still in a0, a1.
__device__ inline float move_reference(Tok &t, f32x4 &a0, f32x4 &a1, u32x4 &pb) {
    float mx = fmaxf(fmaxf(a0[0], a0[1]), a0[2]);
    mx = fmaxf(fmaxf(mx, a0[3]), a1[0]);
    mx = fmaxf(fmaxf(mx, a1[1]), a1[2]);
    mx = fmaxf(mx, a1[3]);
    mx = rows_max(mx);                     // all four lanes of a head agree
    float delta = __builtin_fmaf(mx, t.cm, t.nr);      // by how much the largest exponent exceeds the reference
    float alpha = 1.0f;
    if (t.slack > 0.f) {
        delta = fmaxf(delta, 0.f);         // never down once there is history
        alpha = fast_exp2(-delta);
    }
    t.slack = kSumSlack;
    t.nr -= delta;
    t.l *= alpha;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) t.o[dt] *= alpha;
    float ls = 0.f, p[2];
#pragma unroll
    for (int e = 0; e < 8; ++e) ls += prob_step<false>(a0, a1, e, p, pb, t.cm, t.nr, 0, 0);
    return ls;
}

// One token against one block.  OWN: the block is the token's own and keys past key_limit are masked.
//
// The block is handled as two halves of 32 keys so that the vector work of the softmax always has matrix work
// of the same wave to hide under: the exponentials of the first half are issued between the S^T products of the
// second half, those of the second half between the PV products of the first.  (With the whole block's softmax
// between the two groups of products, the waves of a workgroup, which start every unit together after a barrier,
// all reach the softmax at the same time and the matrix core idles meanwhile.)  The order below is the issue
// order: a scheduling fence after every step keeps the compiler from regrouping it.
struct NoMid {
    __device__ inline void operator()() const {}
};

// `mid` is called once, after the second group of products (the S^T half of the unit) has been issued: work of the
// caller that must not delay the start of the unit but should be under way well before its end (the tile kernel
// issues its copies there).
template <bool OWN, class Mid = NoMid>
__device__ inline void unit(Tok &t, uint32_t stage, uint32_t kx, uint32_t vx, int lane, int key_limit, Mid mid = Mid()) {
    const int key0 = 8 * (lane >> 4);
    const uint32_t kb = stage + kx, vb = stage + vx;
    constexpr int W = 4;               // operand fetches run W products ahead, through all four groups of products
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    f32x4 acc[4];
    u32x4 pb[2];
    bf16x8 f[W];
    float p[2];
    // fragment n of the unit: 0-7 K rows of the first half (key tile n & 1, k-step n >> 1), 8-15 of the second
    // half, 16-23 V^T k-step 0 (dim tile n & 7), 24-31 V^T k-step 1
    auto frag = [&](int n) -> bf16x8 {
        if (n < 16) return k_frag(kb, 2 * (n >> 3) + (n & 1), (n >> 1) & 3);
        return v_frag(vb, n & 7, (n >> 3) & 1);
    };
#pragma unroll
    for (int n = 0; n < W; ++n) f[n] = frag(n);
    // Products are issued in pairs, the later-fetched fragment first: LDS reads return in order, so the one wait
    // for that fragment covers the pair (16 waits per unit instead of 32; a lone wave on a SIMD is bound by the
    // number of instructions it has to issue).  The two products of a pair write different accumulators.
    // ---- exponents of the first half (8 products, 2 accumulators)
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
        const int s = i >> 1;
        acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[(i + 1) % W], t.qf[s], s == 0 ? zero : acc[1], 0, 0, 0);
        acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[i % W], t.qf[s], s == 0 ? zero : acc[0], 0, 0, 0);
        f[i % W] = frag(i + W);
        f[(i + 1) % W] = frag(i + 1 + W);
        __builtin_amdgcn_sched_barrier(0);
    }
    // ---- second half's exponents || first half's probabilities
    float ls = 0.f;
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
        const int s = i >> 1;
        acc[3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[(8 + i + 1) % W], t.qf[s], s == 0 ? zero : acc[3], 0, 0, 0);
        acc[2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[(8 + i) % W], t.qf[s], s == 0 ? zero : acc[2], 0, 0, 0);
        f[(8 + i) % W] = frag(8 + i + W);
        f[(8 + i + 1) % W] = frag(8 + i + 1 + W);
        ls += prob_step<OWN>(acc[0], acc[1], i, p, pb[0], t.cm, t.nr, key0, key_limit);
        ls += prob_step<OWN>(acc[0], acc[1], i + 1, p, pb[0], t.cm, t.nr, key0, key_limit);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (__any(!(ls < t.slack))) ls = move_reference(t, acc[0], acc[1], pb[0]);
    t.l += ls;
    mid();
    // ---- O^T += V^T P^T of the first half || second half's probabilities
    ls = 0.f;
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
        t.o[i + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[(16 + i + 1) % W], __builtin_bit_cast(bf16x8, pb[0]), t.o[i + 1], 0, 0, 0);
        t.o[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[(16 + i) % W], __builtin_bit_cast(bf16x8, pb[0]), t.o[i], 0, 0, 0);
        f[(16 + i) % W] = frag(16 + i + W);
        f[(16 + i + 1) % W] = frag(16 + i + 1 + W);
        ls += prob_step<OWN>(acc[2], acc[3], i, p, pb[1], t.cm, t.nr, key0 + 32, key_limit);
        ls += prob_step<OWN>(acc[2], acc[3], i + 1, p, pb[1], t.cm, t.nr, key0 + 32, key_limit);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (__any(!(ls < t.slack))) ls = move_reference(t, acc[2], acc[3], pb[1]);
    t.l += ls;
    // ---- second half
#pragma unroll
    for (int i = 0; i < 8; i += 2) {
        t.o[i + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[(24 + i + 1) % W], __builtin_bit_cast(bf16x8, pb[1]), t.o[i + 1], 0, 0, 0);
        t.o[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(f[(24 + i) % W], __builtin_bit_cast(bf16x8, pb[1]), t.o[i], 0, 0, 0);
        if (i + W < 8) {
            f[(24 + i) % W] = frag(24 + i + W);
            f[(24 + i + 1) % W] = frag(24 + i + 1 + W);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

}  // namespace attn_unit
}  // namespace ifv2
