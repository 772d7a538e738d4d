// Instantiation of the fp16 MFMA GEMM: 256 x 256 workgroup tile, 8 wavefronts.
#include "gemm_mfma_impl.h"
namespace zs {
hipError_t gemm_mfma_256x256_f16(hipStream_t st, const Gemm& g) { return gemm_impl::gemm_mfma_tile<f16, 256, 256, 8>(st, g); }
}  // namespace zs
