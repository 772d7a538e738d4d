// What the matrix cores sustain with nothing else going on: a loop of MFMAs on operands that stay in registers (random
// values, changing from one instruction to the next as in a GEMM's inner loop), no LDS and no memory traffic inside
// the loop, on the register footprint of the GEMM's 128 x 64 wave tile (128 accumulator registers, two waves per SIMD,
// one workgroup per CU).  The chip runs such a loop at its power limit, so the result is the ceiling that a bf16 GEMM
// can approach on this hardware, and it depends on the instruction shape.
#include "kernels.h"

namespace zs {
namespace {

__global__ __launch_bounds__(512, 1) void mfma_rate_32x32x16(const bf16x8* __restrict__ src, float* __restrict__ sink, int iters) {
  bf16x8 a[2][4], b[2][2];
  for (int s = 0; s < 2; ++s) {
    for (int i = 0; i < 4; ++i) a[s][i] = src[(threadIdx.x * 16 + s * 4 + i) % 4096];
    for (int j = 0; j < 2; ++j) b[s][j] = src[(threadIdx.x * 16 + 8 + s * 2 + j) % 4096];
  }
  f32x16 acc[4][2];
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 2; ++j) for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {   // 16 MFMAs = 32 columns of k per iteration
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[s][j], a[s][i], acc[i][j], 0, 0, 0);
  }
  float t = 0.f;
  for (int i = 0; i < 4; ++i) for (int j = 0; j < 2; ++j) for (int r = 0; r < 16; ++r) t += acc[i][j][r];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = t;
}

__global__ __launch_bounds__(512, 1) void mfma_rate_16x16x32(const bf16x8* __restrict__ src, float* __restrict__ sink, int iters) {
  bf16x8 a[8], b[4];
  for (int i = 0; i < 8; ++i) a[i] = src[(threadIdx.x * 16 + i) % 4096];
  for (int j = 0; j < 4; ++j) b[j] = src[(threadIdx.x * 16 + 8 + j) % 4096];
  f32x4 acc[8][4];
  for (int i = 0; i < 8; ++i) for (int j = 0; j < 4; ++j) for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {   // 32 MFMAs = 32 columns of k per iteration
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
  }
  float t = 0.f;
  for (int i = 0; i < 8; ++i) for (int j = 0; j < 4; ++j) for (int r = 0; r < 4; ++r) t += acc[i][j][r];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = t;
}

}  // namespace

hipError_t mfma_rate(hipStream_t st, int shape, int iters, const void* operands, float* sink) {
  if (shape == 16) hipLaunchKernelGGL(mfma_rate_16x16x32, dim3(MFMA_RATE_BLOCKS), dim3(512), 0, st, (const bf16x8*)operands, sink, iters);
  else hipLaunchKernelGGL(mfma_rate_32x32x16, dim3(MFMA_RATE_BLOCKS), dim3(512), 0, st, (const bf16x8*)operands, sink, iters);
  return hipGetLastError();
}

}  // namespace zs
