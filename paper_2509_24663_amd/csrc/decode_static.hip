// infllmv2_sparse_decode_static: the decode step for callers that cannot allocate or own device scratch (code under
// HIP graph capture that may not call hipMalloc, tight serving loops, harnesses that forbid allocation).  It is
// infllmv2_sparse_decode with the workspace argument replaced by a fixed array in the library's own device image.
#include <atomic>

#include "common.h"

namespace {

constexpr size_t kScratchBytes = (size_t)16 << 20;      // 16 MiB: config-4-sized steps (batch 16, contexts to 65536)

// One copy per GPU the library runs on, at its own address on each, held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress: the address kernels can use is what that call returns.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::atomic<void *> scratch_ptr[kMaxDevices];           // device address of `scratch` on each GPU, once looked up

// Address of this GPU's copy of the array (looked up on the first call with this device current).  Two threads
// that race here both store the same value.
int scratch_address(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return INFLLMV2_ERR_HIP;
    void *ptr = scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return INFLLMV2_ERR_HIP;
        scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return INFLLMV2_OK;
}

}  // namespace

extern "C" {

size_t infllmv2_sparse_decode_static_capacity(void) { return kScratchBytes; }

int infllmv2_sparse_decode_static(const infllmv2_params *p, const void *q_d, const void *k_cache_d, const void *v_cache_d,
                                  int64_t kv_batch_stride, int64_t kv_head_stride, int64_t kv_tok_stride,
                                  const float *kc_cache_d, int64_t kc_head_stride, const int32_t *ctx_lens_h,
                                  const int32_t *ctx_lens_d, int32_t batch, int32_t *block_idx_out_d, void *out_d,
                                  float *lse_d, void *stream) {
    if (p == nullptr || ctx_lens_h == nullptr || batch < 0) return INFLLMV2_ERR_INVALID_ARGUMENT;
    int32_t max_ctx = 0;
    for (int b = 0; b < batch; ++b) {
        if (ctx_lens_h[b] < 1) return INFLLMV2_ERR_INVALID_ARGUMENT;
        if (ctx_lens_h[b] > max_ctx) max_ctx = ctx_lens_h[b];
    }
    // the step must fit the fixed array: decided on the host, before the device is touched
    const size_t need = infllmv2_decode_workspace_bytes(p, batch, max_ctx);
    if (need > kScratchBytes) return INFLLMV2_ERR_WORKSPACE_TOO_SMALL;
    void *ptr = nullptr;
    if (batch > 0 && need > 0) {
        const int st = scratch_address(&ptr);
        if (st != INFLLMV2_OK) return st;
    }
    // Nothing in the array has to start at zero: every kernel of the step writes what a later one reads.
    return infllmv2_sparse_decode(p, q_d, k_cache_d, v_cache_d, kv_batch_stride, kv_head_stride, kv_tok_stride,
                                  kc_cache_d, kc_head_stride, ctx_lens_h, ctx_lens_d, batch, block_idx_out_d, out_d,
                                  lse_d, ptr, kScratchBytes, stream);
}

}  // extern "C"
