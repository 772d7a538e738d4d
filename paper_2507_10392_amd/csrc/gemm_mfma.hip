// bf16 MFMA GEMM (placeholder until the tiled kernel lands: reports "not supported").
#include "kernels.h"
namespace zs {
bool gemm_mfma_supported(DType, const Gemm&) { return false; }
hipError_t gemm_mfma(hipStream_t, const Gemm&) { return hipErrorNotSupported; }
}  // namespace zs
