// Instantiation of the fp16 MFMA GEMM: 128 x 128 workgroup tile, 4 wavefronts.
#include "gemm_mfma_impl.h"
namespace zs {
hipError_t gemm_mfma_128x128_f16(hipStream_t st, const Gemm& g) { return gemm_impl::gemm_mfma_tile<f16, 128, 128, 4>(st, g); }
}  // namespace zs
