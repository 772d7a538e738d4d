// Cost of an LDS access pattern: every wave of one 512-thread workgroup issues the same wave-wide read (16 bytes per
// lane, or the 8-byte transposing read of gfx950) at the byte offsets given per lane, `iters` x 8 times, and the
// workgroup's cycle count is reported.  Bank conflicts show as cycles per wave read above the pattern-free minimum
// (4.6 for 16-byte reads, 3.6 for transposing reads).  This is how the slab layouts of the GEMM were chosen: the LDS
// does not serve a wave's accesses in groups of 16 consecutive lanes, so a layout has to be timed, not derived.
#include "kernels.h"

namespace zs {
namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
constexpr int LDS_PROBE_BYTES = 65536;

template <int KIND> struct ProbeWord;
template <> struct ProbeWord<0> {
  typedef u32x4 type;
  static __device__ __forceinline__ type read(const char* p) { return *reinterpret_cast<const u32x4*>(p); }
};
template <> struct ProbeWord<1> {
  typedef s16x4 type;
  static __device__ __forceinline__ type read(const char* p) { return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p); }
};

template <int KIND>
__global__ __launch_bounds__(512) void lds_probe_kernel(const int* __restrict__ lane_offset, int iters, long long* __restrict__ cycles) {
  typedef typename ProbeWord<KIND>::type W;
  __shared__ __align__(16) char smem[LDS_PROBE_BYTES];
  for (int i = threadIdx.x; i < LDS_PROBE_BYTES / 4; i += 512) reinterpret_cast<int*>(smem)[i] = i;
  __syncthreads();
  const int a = lane_offset[threadIdx.x & 63];
  W acc[8];
  for (int u = 0; u < 8; ++u) acc[u] = W{0, 0, 0, 0};
  __syncthreads();
  const long long t0 = clock64();
  for (int it = 0; it < iters; ++it) {
    W v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)   // eight independent reads in flight; the uniform shifts do not change the bank pattern
      v[u] = ProbeWord<KIND>::read(smem + a + ((it & 3) << 12) + u * 4608);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      asm volatile("" : "+v"(v[u]));
      acc[u] ^= v[u];
    }
  }
  __syncthreads();
  const long long t1 = clock64();
  W t = acc[0];
  for (int u = 1; u < 8; ++u) t ^= acc[u];
  if (threadIdx.x == 0) {
    cycles[0] = t1 - t0;
    cycles[1] = (long long)(t[0] ^ t[1] ^ t[2] ^ t[3]);   // keeps the reads alive
  }
}

}  // namespace

// Largest byte offset a lane may pass: the probe adds up to 3 * 4096 + 7 * 4608 bytes of uniform shifts and reads 16 bytes.
int lds_probe_max_offset() { return LDS_PROBE_BYTES - 3 * 4096 - 7 * 4608 - 16; }

hipError_t lds_probe(hipStream_t st, int kind, const int* lane_offset, int iters, long long* cycles) {
  if (kind == 0) hipLaunchKernelGGL(lds_probe_kernel<0>, dim3(1), dim3(512), 0, st, lane_offset, iters, cycles);
  else hipLaunchKernelGGL(lds_probe_kernel<1>, dim3(1), dim3(512), 0, st, lane_offset, iters, cycles);
  return hipGetLastError();
}

}  // namespace zs
