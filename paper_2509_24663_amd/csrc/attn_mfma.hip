// bf16 MFMA attention kernels (placeholder until the tile kernel lands).
#include "common.h"
namespace ifv2 {
bool attn_mfma_supported(const infllmv2_params *) { return false; }
int launch_attn_mfma(const Launch &, const void *, const void *, const void *, const int32_t *, int, void *, float *,
                     const int32_t *) {
    return INFLLMV2_ERR_UNSUPPORTED;
}
}  // namespace ifv2
