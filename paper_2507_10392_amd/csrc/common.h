// Shared device/host helpers for the stage kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace zs {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum DType { F32 = 0, BF16 = 1, F16 = 2 };   // F16: IEEE half (the precision the paper trains in, Section 6.1)

constexpr int WAVE = 64;

__device__ __forceinline__ float to_f(float x) { return x; }
__device__ __forceinline__ float to_f(bf16 x) { return (float)x; }
__device__ __forceinline__ float to_f(f16 x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f(float x);
template <> __device__ __forceinline__ float from_f<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f<bf16>(float x) { return (bf16)x; }  // round-to-nearest-even
template <> __device__ __forceinline__ f16 from_f<f16>(float x) { return (f16)x; }     // round-to-nearest-even, overflow to inf

// Elements moved per 16-byte access.
template <typename T> struct Vec;
template <> struct Vec<float> { static constexpr int N = 4; typedef f32x4 type; };
template <> struct Vec<bf16> { static constexpr int N = 8; typedef bf16x8 type; };
template <> struct Vec<f16> { static constexpr int N = 8; typedef f16x8 type; };

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Sum over a workgroup of NW waves; every thread gets the result.  red must hold NW floats.
template <int NW> __device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  __syncthreads();
  if (l == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) t += red[i];
  return t;
}

// Gated FFN unit of the Llama-style layer: a = silu(gate) * up, and (dgate, dup) from da.  One definition, so that
// the stand-alone kernels and the GEMM epilogues that fuse them produce the same bits.
// exp through the hardware's exp2 and a hardware reciprocal (each good to about one fp32 ulp, far below the 16-bit
// rounding of whatever is stored): a fifth of the instructions of expf and an IEEE division, which matters where this runs
// 65 536 times in the store phase of a GEMM tile with the matrix cores waiting.
__device__ __forceinline__ float sigmoid_f(float z) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
}
__device__ __forceinline__ float glu_f(float g, float u) { return g * sigmoid_f(g) * u; }
__device__ __forceinline__ void glu_df(float d, float g, float u, float& dg, float& du) {
  const float s = sigmoid_f(g);
  du = d * g * s;
  dg = d * u * s * (1.0f + g * (1.0f - s));
}

static inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace zs
