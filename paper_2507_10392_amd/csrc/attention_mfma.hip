// bf16 MFMA flash attention (placeholder until the tiled kernel lands: reports "not supported").
#include "kernels.h"
namespace zs {
bool attn_mfma_supported(DType, int, int) { return false; }
hipError_t attn_fwd_mfma(hipStream_t, int, int, int, int, const void*, const void*, const void*, int64_t, void*, int64_t,
                         float*) { return hipErrorNotSupported; }
hipError_t attn_bwd_mfma(hipStream_t, int, int, int, int, const void*, const void*, const void*, int64_t, const void*,
                         const void*, int64_t, const float*, float*, void*, void*, void*, int64_t) {
  return hipErrorNotSupported;
}
}  // namespace zs
