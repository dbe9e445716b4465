// Stage 3 kernel: one wavefront per (token, KV head) row; the selection itself is in topk_row.h.
#include "topk_row.h"

namespace ifv2 {

// NCH > 0: pooled keys live in NCH registers per lane; NCH == 0: in LDS.
template <int NCH, int MODE>
__global__ void __launch_bounds__(256)
topk_blocks_kernel(const float *__restrict__ s_shared, int64_t row_stride, RowMap map, TopkArgs a,
                   int32_t *__restrict__ idx, int lds_keys_per_wave) {
    extern __shared__ uint32_t lds_keys[];
    __shared__ uint2 cand[NCH > kCandChunks ? 4 * kCandPerWave : 1];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int row = blockIdx.x * 4 + w, h = blockIdx.y;
    if (row >= map.total_rows) return;
    const RowLoc loc = locate(map, row);
    int32_t *out = idx + head_row(map, h, row) * a.topk_total;
    if (loc.len < a.dense_below) {
        for (int j = lane; j < a.topk_total; j += 64) out[j] = -1;
        return;
    }
    topk_row<NCH, MODE>(s_shared + head_row(map, h, row) * row_stride, loc.pos, a, out,
                  lds_keys + (size_t)w * lds_keys_per_wave, cand + (NCH > kCandChunks ? w * kCandPerWave : 0), lane);
}

template <int NCH>
static int launch_n(const Launch &L, const float *s, int64_t rs, int32_t *idx, const TopkArgs &a, size_t lds, int per_wave,
                    bool pooled) {
    dim3 grid((L.map.total_rows + 3) / 4, L.p->num_kv_heads);
    if (grid.x == 0) return INFLLMV2_OK;
    const bool fast = NCH > 0 && a.pool_len == 5 && a.pool_stride == 4 && a.pool_pad == 0 && rs % 4 == 0 &&
                      ((uintptr_t)s & 15) == 0;
    if (pooled)
        hipLaunchKernelGGL((topk_blocks_kernel<NCH, TOPK_POOLED>), grid, dim3(256), lds, L.stream, s, rs, L.map, a, idx, per_wave);
    else if (fast)
        hipLaunchKernelGGL((topk_blocks_kernel<NCH, TOPK_POOL_FAST>), grid, dim3(256), lds, L.stream, s, rs, L.map, a, idx, per_wave);
    else
        hipLaunchKernelGGL((topk_blocks_kernel<NCH, TOPK_POOL_ANY>), grid, dim3(256), lds, L.stream, s, rs, L.map, a, idx, per_wave);
    return hip_status(hipGetLastError());
}

int launch_topk(const Launch &L, const float *s_shared, int64_t row_stride, int32_t *idx, bool pooled) {
    const infllmv2_params *p = L.p;
    TopkArgs a{p->cmp_len, p->cmp_stride, p->pool_len, p->pool_stride, p->pool_pad, p->n_init, p->n_local, p->topk_total,
               p->dense_threshold};
    const int max_blocks = (L.max_len + kBlock - 1) / kBlock;
    const int nch = (max_blocks + 63) / 64;
    if (nch <= 4) return launch_n<4>(L, s_shared, row_stride, idx, a, 0, 0, pooled);
    if (nch <= 8) return launch_n<8>(L, s_shared, row_stride, idx, a, 0, 0, pooled);
    if (nch <= 16) return launch_n<16>(L, s_shared, row_stride, idx, a, 0, 0, pooled);
    if (nch <= 32) return launch_n<32>(L, s_shared, row_stride, idx, a, 0, 0, pooled);
    const int per_wave = nch * 64;
    const size_t lds = (size_t)per_wave * 4 * sizeof(uint32_t);
    if (lds > 64 * 1024) return INFLLMV2_ERR_UNSUPPORTED;     // > 262144 tokens per sequence
    return launch_n<0>(L, s_shared, row_stride, idx, a, lds, per_wave, pooled);
}

}  // namespace ifv2
