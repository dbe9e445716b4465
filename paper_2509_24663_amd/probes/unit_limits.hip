// Measurements behind the roofline model of the prefill attention kernel and of decode (one MI355X, no inputs):
//   1. the issue mix of a (token, block) attention unit -- matrix products whose A operand streams in from LDS, with
//      and without the softmax's vector work -- as clocks per 16x16x32 product and SIMD, for 1, 2 and 4 waves per SIMD;
//   2. the attention unit of the library itself (attn_unit.h) run back to back on a resident LDS stage: time per unit
//      of one wave (its latency) and per SIMD (throughput) for 1, 2 and 4 waves per SIMD;
//   3. how fast a burst of N bytes streams from HBM, cold (rotating buffers) and warm, and what an empty dependent
//      launch costs;
//   4. batches of global -> LDS copies as the attention kernel issues them (one workgroup of 16 waves per CU, B KB
//      requested at once as 1 KB pieces from scattered 16 KB blocks, then waited for): time per batch against the
//      bytes in flight, from a span that misses the caches, one that fits the memory-side cache and one that stays in L2.
// Build: hipcc --offload-arch=gfx950 -O3 -std=c++17 -I include -I paper_2509_24663_amd/csrc
//        -o paper_2509_24663_amd/probes/unit_limits paper_2509_24663_amd/probes/unit_limits.hip
// (python paper_2509_24663_amd/build.py --probes does it).  Clocks are counted at the nominal 2.4 GHz.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include <vector>

#include "attn_unit.h"

using namespace ifv2;
using namespace ifv2::attn_unit;

#define CHECK(x)                                                                            \
    do {                                                                                    \
        hipError_t e_ = (x);                                                                \
        if (e_ != hipSuccess) {                                                             \
            fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));                  \
            return 1;                                                                       \
        }                                                                                   \
    } while (0)

constexpr double kClockHz = 2.4e9;

// ---------------------------------------------------------------------------------------------- 1. issue mix
// per group: R 16-byte-per-lane LDS reads, M products, V fused multiply-adds, X exponentials
template <int R, int M, int V, int X>
__global__ void __launch_bounds__(1024) mix_kernel(float *out, int iters) {
    extern __shared__ __attribute__((aligned(1024))) uint16_t lds[];
    for (int i = threadIdx.x; i < 32768; i += blockDim.x) lds[i] = (uint16_t)(0x3c00 + (i & 63));
    __syncthreads();
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint16_t *base = lds + lane * 8;
    f32x4 acc[8];
    for (int i = 0; i < 8; ++i) acc[i] = f32x4{0, 0, 0, 0};
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = lane * 1e-3f + i;
    bf16x8 b;
    for (int i = 0; i < 8; ++i) b[i] = (__bf16)(1.0f + lane * 0.01f);
    int off = w * 512;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            bf16x8 a[R > 0 ? R : 1];
            if (R == 0) a[0] = b;
#pragma unroll
            for (int r = 0; r < R; ++r) a[r] = *reinterpret_cast<const bf16x8 *>(base + ((off + (g * R + r) * 512) & 32767 & ~511));
#pragma unroll
            for (int m = 0; m < M; ++m)
                acc[(g * M + m) & 7] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[R > 0 ? m % R : 0], b, acc[(g * M + m) & 7], 0, 0, 0);
            if (M == 0) {
#pragma unroll
                for (int r = 0; r < R; ++r) asm volatile("" ::"v"(a[r]));
            }
#pragma unroll
            for (int v = 0; v < V; ++v) x[(g * V + v) & 7] = x[(g * V + v) & 7] * 0.999f + 0.5f;
#pragma unroll
            for (int e = 0; e < X; ++e) x[(g * X + e + 4) & 7] = __builtin_amdgcn_exp2f(x[(g * X + e + 4) & 7]);
        }
        off += 8 * (R > 0 ? R : 1) * 512 + 512;
    }
    float s = 0;
    for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][3] + x[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The same with 32x32x16 products (two tokens' 16 heads as the 32 columns): one 1 KB fragment feeds a product that
// keeps the matrix core twice as long, and carries two tokens' vector work.  256 registers: 1 or 2 waves per SIMD.
typedef float f32x16 __attribute__((ext_vector_type(16)));
template <int R, int M, int V, int X>
__global__ void __launch_bounds__(512) mix32_kernel(float *out, int iters) {
    extern __shared__ __attribute__((aligned(1024))) uint16_t lds[];
    for (int i = threadIdx.x; i < 32768; i += blockDim.x) lds[i] = (uint16_t)(0x3c00 + (i & 63));
    __syncthreads();
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const uint16_t *base = lds + lane * 8;
    f32x16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = lane * 1e-3f + i;
    bf16x8 b;
    for (int i = 0; i < 8; ++i) b[i] = (__bf16)(1.0f + lane * 0.01f);
    int off = w * 512;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            bf16x8 a[R];
#pragma unroll
            for (int r = 0; r < R; ++r) a[r] = *reinterpret_cast<const bf16x8 *>(base + ((off + (g * R + r) * 512) & 32767 & ~511));
#pragma unroll
            for (int m = 0; m < M; ++m)
                acc[(g * M + m) & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[m % R], b, acc[(g * M + m) & 3], 0, 0, 0);
#pragma unroll
            for (int v = 0; v < V; ++v) x[(g * V + v) & 7] = x[(g * V + v) & 7] * 0.999f + 0.5f;
#pragma unroll
            for (int e = 0; e < X; ++e) x[(g * X + e + 4) & 7] = __builtin_amdgcn_exp2f(x[(g * X + e + 4) & 7]);
        }
        off += 8 * R * 512 + 512;
    }
    float s = 0;
    for (int i = 0; i < 4; ++i) s += acc[i][0] + acc[i][15];
    for (int i = 0; i < 8; ++i) s += x[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int R, int M, int V, int X>
int run_mix32(const char *name, float *d) {
    const int iters = 2048, lds = 96 * 1024;
    auto kf = mix32_kernel<R, M, V, X>;
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kf), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    printf("%-44s", name);
    for (int nw : {4, 8}) {
        hipLaunchKernelGGL(kf, dim3(512), dim3(nw * 64), lds, 0, d, iters);
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL(kf, dim3(512), dim3(nw * 64), lds, 0, d, iters);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        const double clks = ms * 1e-3 * kClockHz / 2.0;
        const double per_group = clks / (iters * 8.0 * (nw / 4));
        // a 32x32x16 product is worth two 16x16x32 ones: 32 clocks at peak
        printf(" | %d w/SIMD %5.1f clk per 32x32x16 product (%4.1f%% of peak)", nw / 4, per_group / M, 100.0 * M * 32.0 / per_group);
    }
    printf("\n");
    fflush(stdout);
    return 0;
}

template <int R, int M, int V, int X>
int run_mix(const char *name, float *d) {
    const int iters = 2048, lds = 96 * 1024;         // 96 KB of LDS: one workgroup per CU
    auto kf = mix_kernel<R, M, V, X>;
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kf), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    printf("%-44s", name);
    for (int nw : {4, 8, 16}) {
        hipLaunchKernelGGL(kf, dim3(512), dim3(nw * 64), lds, 0, d, iters);
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL(kf, dim3(512), dim3(nw * 64), lds, 0, d, iters);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        const double clks = ms * 1e-3 * kClockHz / 2.0;                  // two workgroups per CU, one after the other
        const double per_group = clks / (iters * 8.0 * (nw / 4));        // SIMD clocks per group
        if (M > 0) printf(" | %d w/SIMD %5.1f clk/product (%4.1f%% of peak)", nw / 4, per_group / M, 100.0 * M * 16.0 / per_group);
        else printf(" | %d w/SIMD %5.1f clk/group, %5.1f B/clk/CU  ", nw / 4, per_group, R * 1024.0 * 4 / per_group);
    }
    printf("\n");
    fflush(stdout);
    return 0;
}

// ---------------------------------------------------------------------------------------------- 2. the unit itself
__global__ void __launch_bounds__(1024) unit_kernel(float *out, int units) {
    extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
    // a plausible stage: small bf16 values everywhere (K tile, then V^T tile)
    for (int i = threadIdx.x; i < STAGE_ELEMS; i += blockDim.x) smem[i] = (uint16_t)(0x3c00 + ((i * 7) & 127));
    __syncthreads();
    const int lane = threadIdx.x & 63;
    Tok st;
    float cm;
    int ce;
    split_scale(0.0883883f * LOG2E, cm, ce);
    for (int s = 0; s < 4; ++s) {
        uint4 raw = make_uint4(0x3c003c00u + lane, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u);
        st.qf[s] = scale_q(raw, ce);
    }
    tok_init(st, cm);
    const uint32_t stage = lds_address(smem);
    const uint32_t kx = k_lane_bytes(lane), vx = v_lane_bytes(lane);
    for (int u = 0; u < units; ++u) unit<false>(st, stage, kx, vx, lane, 0);
    float s = st.l;
    for (int dt = 0; dt < 8; ++dt) s += st.o[dt][0] + st.o[dt][3];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

int run_unit(float *d) {
    const int units = 4096, lds = 96 * 1024;
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(unit_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    printf("%-44s", "attention unit (token x 64-key block)");
    for (int nw : {4, 8, 16}) {
        hipLaunchKernelGGL(unit_kernel, dim3(512), dim3(nw * 64), lds, 0, d, units);
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL(unit_kernel, dim3(512), dim3(nw * 64), lds, 0, d, units);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        const double clks = ms * 1e-3 * kClockHz / 2.0;
        const double per_wave = clks / units, per_simd = per_wave / (nw / 4);
        printf(" | %d w/SIMD: %6.0f clk per unit of a wave, %6.0f per unit and SIMD (%4.1f%% of peak)", nw / 4, per_wave,
               per_simd, 100.0 * 32 * 16.0 / per_simd);
    }
    printf("\n");
    fflush(stdout);
    return 0;
}

// ---------------------------------------------------------------------------------------------- 3. streaming
template <int U>
__global__ void __launch_bounds__(256) stream_kernel(const float4 *__restrict__ p, size_t n4, float *out) {
    const size_t base = (size_t)blockIdx.x * (U * 256) + threadIdx.x;
    float4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t i = base + (size_t)u * 256;
        v[u] = i < n4 ? p[i] : make_float4(0, 0, 0, 0);
    }
    float s = 0;
#pragma unroll
    for (int u = 0; u < U; ++u) s += v[u].x + v[u].y + v[u].z + v[u].w;
    if (s == 12345.678f) out[0] = s;
}

int run_stream(std::vector<float4 *> &bufs, size_t bytes, float *out, bool cold) {
    constexpr int U = 4;
    const size_t n4 = bytes / 16;
    const unsigned grid = (unsigned)((n4 + U * 256 - 1) / (U * 256));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const int reps = 16;
    for (int i = 0; i < 4; ++i) hipLaunchKernelGGL(stream_kernel<U>, dim3(grid), dim3(256), 0, 0, bufs[cold ? i % bufs.size() : 0], n4, out);
    CHECK(hipEventRecord(e0));
    for (int i = 0; i < reps; ++i)
        hipLaunchKernelGGL(stream_kernel<U>, dim3(grid), dim3(256), 0, 0, bufs[cold ? (i + 4) % bufs.size() : 0], n4, out);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double us = ms * 1e3 / reps;
    printf("stream %s %7.1f MB: %7.2f us per launch (back to back), %5.2f TB/s\n", cold ? "cold" : "warm", bytes / 1e6, us,
           bytes / us * 1e-6);
    fflush(stdout);
    return 0;
}


// ---------------------------------------------------------------------------------------------- 4. LDS fills
// PPW one-KB pieces per wave and batch (16 waves: 16 PPW KB per batch), each batch from 16-KB blocks chosen by a hash of
// (workgroup, batch, block in batch) inside `span` bytes.
template <int PPW>
__global__ void __launch_bounds__(1024) fill_kernel(const char *src, uint32_t span_blocks, int batches, float *out) {
    extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
    for (int b = 0; b < batches; ++b) {
#pragma unroll
        for (int p = 0; p < PPW; ++p) {
            const int q = w * PPW + p;                          // piece of the batch
            const uint32_t blk = ((uint32_t)blockIdx.x * 2654435761u + (uint32_t)b * 40503u + (uint32_t)(q >> 4) * 2246822519u) % span_blocks;
            const char *base = src + (size_t)blk * 16384 + (size_t)(q & 15) * 1024;
            async_copy16(base, (uint32_t)lane * 16u, lds0 + (uint32_t)q * 1024u);
        }
        __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
        __syncthreads();
    }
    if (out != nullptr && threadIdx.x == 0) out[blockIdx.x] = (float)smem[lane];
}

template <int PPW>
int run_fill(const char *src, size_t span_bytes, float *out, const char *what) {
    const int batches = 400, lds = 16 * PPW * 1024;
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(fill_kernel<PPW>), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const uint32_t span_blocks = (uint32_t)(span_bytes / 16384);
    hipLaunchKernelGGL(fill_kernel<PPW>, dim3(256), dim3(1024), lds, 0, src, span_blocks, batches, out);
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL(fill_kernel<PPW>, dim3(256), dim3(1024), lds, 0, src, span_blocks, batches, out);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double us = ms * 1e3 / batches, kb = 16.0 * PPW;
    printf("fills %-22s %4.0f KB per batch and CU: %6.2f us per batch, %5.1f GB/s per CU, %5.2f TB/s over 256 CUs\n", what, kb, us,
           kb * 1024 / us * 1e-3, kb * 1024 * 256 / us * 1e-6);
    fflush(stdout);
    return 0;
}

// The same 64 KB batches (into the upper half of a 128 KB buffer) while NU of the 16 waves run one attention unit per
// batch on the lower half, as in the attention kernel: do the copies and the units' LDS reads get in each other's way?
// NCW < 16: the copies are issued by the last NCW waves alone (64 / NCW pieces each), which run no unit.
template <int NU, int UPB = 1, bool BARRIER = true, int NCW = 16>
__global__ void __launch_bounds__(1024) fill_unit_kernel(const char *src, uint32_t span_blocks, int batches, int copies, float *out) {
    extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
    for (int i = threadIdx.x; i < 2 * STAGE_ELEMS; i += blockDim.x) smem[i] = (uint16_t)(0x3c00 + ((i * 7) & 127));
    __syncthreads();
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
    Tok st;
    float cm;
    int ce;
    split_scale(0.0883883f * LOG2E, cm, ce);
    for (int s = 0; s < 4; ++s) st.qf[s] = scale_q(make_uint4(0x3c003c00u + lane, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u), ce);
    tok_init(st, cm);
    const uint32_t kx = k_lane_bytes(lane), vx = v_lane_bytes(lane);
    // the NU busy waves are spread over the four SIMDs (wave w sits on SIMD w % 4 of a 16-wave workgroup)
    const bool busy = w < NU;
    for (int b = 0; b < batches; ++b) {
        if (copies && NCW == 16) {
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const int q = w * 4 + p;
                const uint32_t blk = ((uint32_t)blockIdx.x * 2654435761u + (uint32_t)b * 40503u + (uint32_t)(q >> 4) * 2246822519u) % span_blocks;
                const char *base = src + (size_t)blk * 16384 + (size_t)(q & 15) * 1024;
                async_copy16(base, (uint32_t)lane * 16u, lds0 + (uint32_t)(2 * STAGE_ELEMS * 2) + (uint32_t)q * 1024u);
            }
        }
        if (copies && NCW < 16 && w >= 16 - NCW) {
#pragma unroll
            for (int q = w - (16 - NCW); q < 64; q += NCW) {
                const uint32_t blk = ((uint32_t)blockIdx.x * 2654435761u + (uint32_t)b * 40503u + (uint32_t)(q >> 4) * 2246822519u) % span_blocks;
                const char *base = src + (size_t)blk * 16384 + (size_t)(q & 15) * 1024;
                async_copy16(base, (uint32_t)lane * 16u, lds0 + (uint32_t)(2 * STAGE_ELEMS * 2) + (uint32_t)q * 1024u);
            }
        }
        if (busy) {
#pragma unroll 1
            for (int u = 0; u < UPB; ++u) unit<false>(st, lds0 + (uint32_t)((b & 1) * STAGE_ELEMS * 2), kx, vx, lane, 0);
        }
        __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
        if (BARRIER) __syncthreads();
    }
    float s = st.l;
    for (int dt = 0; dt < 8; ++dt) s += st.o[dt][0] + st.o[dt][3];
    if (out != nullptr) out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int NU, int UPB = 1, bool BARRIER = true, int NCW = 16>
int run_fill_unit(const char *src, size_t span_bytes, float *out, const char *what) {
    const int batches = 400, lds = 128 * 1024;
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&fill_unit_kernel<NU, UPB, BARRIER, NCW>), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const uint32_t span_blocks = (uint32_t)(span_bytes / 16384);
    double us[2];
    for (int copies = 0; copies < 2; ++copies) {
        hipLaunchKernelGGL((fill_unit_kernel<NU, UPB, BARRIER, NCW>), dim3(256), dim3(1024), lds, 0, src, span_blocks, batches, copies, out);
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL((fill_unit_kernel<NU, UPB, BARRIER, NCW>), dim3(256), dim3(1024), lds, 0, src, span_blocks, batches, copies, out);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        us[copies] = ms * 1e3 / batches;
    }
    char who[48] = "";
    if (NCW < 16) snprintf(who, sizeof who, ", copies issued by %d other waves", NCW);
    printf("64 KB batch %-22s beside %2d waves with %d unit(s) each%s%s: %5.2f us per interval (units alone %5.2f us)\n", what, NU, UPB,
           BARRIER ? "" : ", no barrier", who, us[1], us[0]);
    fflush(stdout);
    return 0;
}

// One LDS base (M0) per wave and batch, the four pieces told apart by the instruction's offset field (it advances the
// global and the LDS address alike): does rewriting M0 between a wave's copies slow their issue?
__global__ void __launch_bounds__(1024) fill_imm_kernel(const char *src, uint32_t span_blocks, int batches, float *out) {
    extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
    for (int b = 0; b < batches; ++b) {
        // wave w copies 4 KB: quarter (w & 3) of the 16 KB block number (w >> 2) of the batch
        const uint32_t blk = ((uint32_t)blockIdx.x * 2654435761u + (uint32_t)b * 40503u + (uint32_t)(w >> 2) * 2246822519u) % span_blocks;
        const char *base = src + (size_t)blk * 16384 + (size_t)(w & 3) * 4096;
        const uint32_t lds = lds0 + (uint32_t)w * 4096u, voff = (uint32_t)lane * 16u;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                     "global_load_lds_dwordx4 %1, %2\n\t"
                     "global_load_lds_dwordx4 %1, %2 offset:1024\n\t"
                     "global_load_lds_dwordx4 %1, %2 offset:2048\n\t"
                     "global_load_lds_dwordx4 %1, %2 offset:3072" ::"s"(lds), "v"(voff), "s"(base) : "memory", "m0");
        __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
        __syncthreads();
    }
    if (out != nullptr && threadIdx.x == 0) out[blockIdx.x] = (float)smem[lane];
}

int run_fill_imm(const char *src, size_t span_bytes, float *out, const char *what) {
    const int batches = 400, lds = 64 * 1024;
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const uint32_t span_blocks = (uint32_t)(span_bytes / 16384);
    hipLaunchKernelGGL(fill_imm_kernel, dim3(256), dim3(1024), lds, 0, src, span_blocks, batches, out);
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL(fill_imm_kernel, dim3(256), dim3(1024), lds, 0, src, span_blocks, batches, out);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double us = ms * 1e3 / batches;
    printf("fills %-22s   64 KB per batch and CU, one M0 per wave: %6.2f us per batch, %5.1f GB/s per CU\n", what, us, 65536 / us * 1e-3);
    fflush(stdout);
    return 0;
}

// NCW waves issue the batch's 64 one-KB copies alone, G copies per M0 write (G = 1: an M0 write before every copy; 4 and
// 8: the instruction's offset field tells the copies of a group apart): how fast can one wave issue copies?
template <int NCW, int G>
__global__ void __launch_bounds__(1024) fill_group_kernel(const char *src, uint32_t span_blocks, int batches, float *out) {
    extern __shared__ __attribute__((aligned(1024))) uint16_t smem[];
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem));
    const uint32_t voff = (uint32_t)lane * 16u;
    for (int b = 0; b < batches; ++b) {
        if (w < NCW) {
#pragma unroll
            for (int q = w * (64 / NCW); q < (w + 1) * (64 / NCW); q += G) {     // pieces q .. q + G - 1: same 16 KB block
                const uint32_t blk = ((uint32_t)blockIdx.x * 2654435761u + (uint32_t)b * 40503u + (uint32_t)(q >> 4) * 2246822519u) % span_blocks;
                const char *base = src + (size_t)blk * 16384 + (size_t)(q & 15) * 1024;
                const uint32_t lds = lds0 + (uint32_t)q * 1024u;
                if (G == 1) {
                    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(voff), "s"(base) : "memory", "m0");
                } else if (G == 4) {
                    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                                 "global_load_lds_dwordx4 %1, %2\n\t"
                                 "global_load_lds_dwordx4 %1, %2 offset:1024\n\t"
                                 "global_load_lds_dwordx4 %1, %2 offset:2048\n\t"
                                 "global_load_lds_dwordx4 %1, %2 offset:3072" ::"s"(lds), "v"(voff), "s"(base) : "memory", "m0");
                } else {
                    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"
                                 "global_load_lds_dwordx4 %1, %2 offset:-4096\n\t"
                                 "global_load_lds_dwordx4 %1, %2 offset:-3072\n\t"
                                 "global_load_lds_dwordx4 %1, %2 offset:-2048\n\t"
                                 "global_load_lds_dwordx4 %1, %2 offset:-1024\n\t"
                                 "global_load_lds_dwordx4 %1, %2\n\t"
                                 "global_load_lds_dwordx4 %1, %2 offset:1024\n\t"
                                 "global_load_lds_dwordx4 %1, %2 offset:2048\n\t"
                                 "global_load_lds_dwordx4 %1, %2 offset:3072" ::"s"(lds + 4096u), "v"(voff), "s"(base + 4096) : "memory", "m0");
                }
            }
        }
        __builtin_amdgcn_s_waitcnt(WAIT_VMCNT0);
        __syncthreads();
    }
    if (out != nullptr && threadIdx.x == 0) out[blockIdx.x] = (float)smem[lane];
}

template <int NCW, int G>
int run_fill_group(const char *src, size_t span_bytes, float *out, const char *what) {
    const int batches = 400, lds = 64 * 1024;
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const uint32_t span_blocks = (uint32_t)(span_bytes / 16384);
    hipLaunchKernelGGL((fill_group_kernel<NCW, G>), dim3(256), dim3(1024), lds, 0, src, span_blocks, batches, out);
    CHECK(hipEventRecord(e0));
    hipLaunchKernelGGL((fill_group_kernel<NCW, G>), dim3(256), dim3(1024), lds, 0, src, span_blocks, batches, out);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double us = ms * 1e3 / batches;
    printf("fills %-22s   64 KB per batch and CU issued by %2d waves, %d copies per M0 write: %6.2f us per batch, %5.1f GB/s per CU\n", what,
           NCW, G, us, 65536 / us * 1e-3);
    fflush(stdout);
    return 0;
}

int main() {
    float *d;
    CHECK(hipMalloc(&d, 512 * 1024 * 4));
    printf("== 1. issue mix: clocks per v_mfma_f32_16x16x32_bf16 and SIMD (16 = peak), nominal 2.4 GHz\n");
    if (run_mix<0, 1, 0, 0>("products only", d)) return 1;
    if (run_mix<1, 0, 0, 0>("LDS reads only (16 B per lane)", d)) return 1;
    if (run_mix<1, 1, 0, 0>("1 read : 1 product", d)) return 1;
    if (run_mix<1, 2, 0, 0>("1 read : 2 products", d)) return 1;
    if (run_mix<1, 4, 0, 0>("1 read : 4 products", d)) return 1;
    if (run_mix<0, 2, 3, 1>("0 reads : 2 products + 3 fma + 1 exp", d)) return 1;
    if (run_mix<2, 2, 3, 1>("2 reads : 2 products + 3 fma + 1 exp", d)) return 1;
    if (run_mix<1, 2, 3, 1>("1 read : 2 products + 3 fma + 1 exp", d)) return 1;
    if (run_mix<1, 4, 6, 2>("1 read : 4 products + 6 fma + 2 exp", d)) return 1;
    if (run_mix32<1, 1, 0, 0>("32x32x16: 1 read : 1 product", d)) return 1;
    if (run_mix32<1, 1, 3, 1>("32x32x16: 1 read : 1 product + 3 fma + 1 exp", d)) return 1;
    if (run_mix32<2, 2, 6, 2>("32x32x16: 2 reads : 2 products + 6 fma + 2 exp", d)) return 1;
    printf("== 2. the library's attention unit on a resident LDS stage (32 products per unit: 512 clocks at peak)\n");
    if (run_unit(d)) return 1;
    printf("== 3. streaming reads (256-thread workgroups, 4 x 16 B per thread), 8 rotating buffers when cold\n");
    {
        const size_t big = (size_t)600 << 20;
        std::vector<float4 *> bufs(8);
        for (auto &b : bufs) {
            CHECK(hipMalloc(&b, big));
            CHECK(hipMemset(b, 1, big));
        }
        float *out;
        CHECK(hipMalloc(&out, 4));
        for (size_t mb : {1, 36, 58, 67, 104, 290, 560})
            for (int cold = 1; cold >= 0; --cold)
                if (run_stream(bufs, mb << 20, out, cold)) return 1;
        printf("== 4. batches of global -> LDS copies (one 16-wave workgroup per CU, 1 KB pieces of scattered 16 KB blocks)\n");
        const char *big0 = reinterpret_cast<const char *>(bufs[0]);
        if (run_fill<1>(big0, big, d, "from 600 MB (misses)")) return 1;
        if (run_fill<2>(big0, big, d, "from 600 MB (misses)")) return 1;
        if (run_fill<4>(big0, big, d, "from 600 MB (misses)")) return 1;
        if (run_fill<6>(big0, big, d, "from 600 MB (misses)")) return 1;
        if (run_fill<8>(big0, big, d, "from 600 MB (misses)")) return 1;
        if (run_fill<2>(big0, (size_t)64 << 20, d, "from 64 MB (MALL hits)")) return 1;
        if (run_fill<4>(big0, (size_t)64 << 20, d, "from 64 MB (MALL hits)")) return 1;
        if (run_fill<8>(big0, (size_t)64 << 20, d, "from 64 MB (MALL hits)")) return 1;
        if (run_fill<2>(big0, (size_t)2 << 20, d, "from 2 MB (L2 hits)")) return 1;
        if (run_fill<4>(big0, (size_t)2 << 20, d, "from 2 MB (L2 hits)")) return 1;
        if (run_fill<8>(big0, (size_t)2 << 20, d, "from 2 MB (L2 hits)")) return 1;
        if (run_fill_imm(big0, (size_t)2 << 20, d, "from 2 MB (L2 hits)")) return 1;
        if (run_fill_imm(big0, (size_t)64 << 20, d, "from 64 MB (MALL hits)")) return 1;
        for (size_t span : {(size_t)600 << 20, (size_t)64 << 20, (size_t)2 << 20}) {
            const char *what = span > ((size_t)100 << 20) ? "from 600 MB (misses)" : span > ((size_t)4 << 20) ? "from 64 MB (MALL hits)" : "from 2 MB (L2 hits)";
            if (run_fill_unit<0>(big0, span, d, what)) return 1;
            if (run_fill_unit<4>(big0, span, d, what)) return 1;
            if (run_fill_unit<8>(big0, span, d, what)) return 1;
            if (run_fill_unit<16>(big0, span, d, what)) return 1;
        }
        if (run_fill_unit<4, 2>(big0, (size_t)64 << 20, d, "from 64 MB (MALL hits)")) return 1;
        if (run_fill_unit<4, 4>(big0, (size_t)64 << 20, d, "from 64 MB (MALL hits)")) return 1;
        if (run_fill_unit<4, 1, false>(big0, (size_t)64 << 20, d, "from 64 MB (MALL hits)")) return 1;
        if (run_fill_unit<16, 2>(big0, (size_t)64 << 20, d, "from 64 MB (MALL hits)")) return 1;
        for (size_t span : {(size_t)64 << 20, (size_t)2 << 20}) {
            const char *what = span > ((size_t)4 << 20) ? "from 64 MB (MALL hits)" : "from 2 MB (L2 hits)";
            if (run_fill_group<1, 1>(big0, span, d, what)) return 1;
            if (run_fill_group<1, 4>(big0, span, d, what)) return 1;
            if (run_fill_group<1, 8>(big0, span, d, what)) return 1;
            if (run_fill_group<2, 8>(big0, span, d, what)) return 1;
            if (run_fill_group<4, 1>(big0, span, d, what)) return 1;
            if (run_fill_group<4, 4>(big0, span, d, what)) return 1;
            if (run_fill_group<4, 8>(big0, span, d, what)) return 1;
            if (run_fill_group<8, 8>(big0, span, d, what)) return 1;
            if (run_fill_group<16, 4>(big0, span, d, what)) return 1;
            if (run_fill_unit<0, 1, true, 4>(big0, span, d, what)) return 1;
            if (run_fill_unit<0, 1, true, 3>(big0, span, d, what)) return 1;
            if (run_fill_unit<0, 1, true, 2>(big0, span, d, what)) return 1;
            if (run_fill_unit<0, 1, true, 1>(big0, span, d, what)) return 1;
            if (run_fill_unit<4, 1, true, 3>(big0, span, d, what)) return 1;
            if (run_fill_unit<13, 1, true, 3>(big0, span, d, what)) return 1;
            if (run_fill_unit<12, 1, true, 4>(big0, span, d, what)) return 1;
        }
    }
    return 0;
}
