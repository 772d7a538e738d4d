// Causal softmax attention, forward and backward, one wavefront per query (or key) row, fp32
// arithmetic, no atomics.  This is the path of the fp32 configuration and of head sizes the MFMA
// kernel does not take; it never materialises the S x S matrix (online softmax over tiles of
// 64 keys) but makes no attempt to reuse K/V across rows.
#include "kernels.h"

namespace zs {

constexpr int MAXD = 256;  // head dim limit of this kernel

template <typename T> __device__ __forceinline__ float dot_row(const float* __restrict__ vec, const T* __restrict__ row, int d) {
  constexpr int V = Vec<T>::N;
  float s = 0.f;
  for (int c = 0; c < d; c += V) {
    typename Vec<T>::type r = *reinterpret_cast<const typename Vec<T>::type*>(row + c);
#pragma unroll
    for (int i = 0; i < V; ++i) s += vec[c + i] * to_f(r[i]);
  }
  return s;
}

// grid (ceil(S/4), nh, mb), 256 threads: wave w handles query row blockIdx.x*4+w.
template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_simple(int S, int d, const T* __restrict__ q, const T* __restrict__ k,
                                                       const T* __restrict__ v, int64_t ld, T* __restrict__ o,
                                                       int64_t ldo, float* __restrict__ lse, float scale) {
  __shared__ float qs[4][MAXD];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + w;
  const int h = blockIdx.y, b = blockIdx.z, nh = gridDim.y;
  if (i >= S) return;                       // whole wave leaves together; no block barrier below
  const int64_t tok0 = (int64_t)b * S;
  const T* qi = q + (tok0 + i) * ld + h * d;
  for (int c = lane; c < d; c += 64) qs[w][c] = to_f(qi[c]) * scale;
  __builtin_amdgcn_wave_barrier();
  float m = -INFINITY, l = 0.f;
  float acc[MAXD / 64];
#pragma unroll
  for (int c = 0; c < MAXD / 64; ++c) acc[c] = 0.f;
  for (int j0 = 0; j0 <= i; j0 += 64) {
    const int j = j0 + lane;
    float s = -INFINITY;
    if (j <= i) s = dot_row(qs[w], k + (tok0 + j) * ld + h * d, d);
    const float mn = fmaxf(m, wave_max(s));
    const float p = (j <= i) ? expf(s - mn) : 0.f;
    const float alpha = expf(m - mn);
    l = l * alpha + wave_sum(p);
    m = mn;
#pragma unroll
    for (int c = 0; c < MAXD / 64; ++c) acc[c] *= alpha;
    const int jn = min(64, i - j0 + 1);
    for (int jj = 0; jj < jn; ++jj) {
      const float pj = __shfl(p, jj, 64);
      const T* vr = v + (tok0 + j0 + jj) * ld + h * d;
#pragma unroll
      for (int c = 0; c < MAXD / 64; ++c)
        if (c * 64 + lane < d) acc[c] += pj * to_f(vr[c * 64 + lane]);
    }
  }
  T* oi = o + (tok0 + i) * ldo + h * d;
#pragma unroll
  for (int c = 0; c < MAXD / 64; ++c)
    if (c * 64 + lane < d) oi[c * 64 + lane] = from_f<T>(acc[c] / l);
  if (lane == 0) lse[((int64_t)b * nh + h) * S + i] = m + logf(l);
}

// delta[b,h,i] = sum_c do[i,c] * o[i,c]
template <typename T>
__global__ __launch_bounds__(256) void attn_delta_kernel(int S, int d, const T* __restrict__ o, const T* __restrict__ dout,
                                                         int64_t ldo, float* __restrict__ delta) {
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + w;
  const int h = blockIdx.y, b = blockIdx.z, nh = gridDim.y;
  if (i >= S) return;
  const int64_t off = ((int64_t)b * S + i) * ldo + h * d;
  float s = 0.f;
  for (int c = lane; c < d; c += 64) s += to_f(o[off + c]) * to_f(dout[off + c]);
  s = wave_sum(s);
  if (lane == 0) delta[((int64_t)b * nh + h) * S + i] = s;
}

// dq_i = scale * sum_{j<=i} ds_ij k_j,  ds_ij = p_ij (do_i.v_j - delta_i),  p_ij = exp(scale q_i.k_j - lse_i)
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_simple(int S, int d, const T* __restrict__ q, const T* __restrict__ k,
                                                          const T* __restrict__ v, int64_t ld,
                                                          const T* __restrict__ dout, int64_t ldo,
                                                          const float* __restrict__ lse, const float* __restrict__ delta,
                                                          T* __restrict__ dq, int64_t ldd, float scale) {
  __shared__ float qs[4][MAXD];
  __shared__ float dos[4][MAXD];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + w;
  const int h = blockIdx.y, b = blockIdx.z, nh = gridDim.y;
  if (i >= S) return;
  const int64_t tok0 = (int64_t)b * S;
  for (int c = lane; c < d; c += 64) {
    qs[w][c] = to_f(q[(tok0 + i) * ld + h * d + c]) * scale;
    dos[w][c] = to_f(dout[(tok0 + i) * ldo + h * d + c]);
  }
  __builtin_amdgcn_wave_barrier();
  const float li = lse[((int64_t)b * nh + h) * S + i];
  const float di = delta[((int64_t)b * nh + h) * S + i];
  float acc[MAXD / 64];
#pragma unroll
  for (int c = 0; c < MAXD / 64; ++c) acc[c] = 0.f;
  for (int j0 = 0; j0 <= i; j0 += 64) {
    const int j = j0 + lane;
    float ds = 0.f;
    if (j <= i) {
      const float s = dot_row(qs[w], k + (tok0 + j) * ld + h * d, d);
      const float dp = dot_row(dos[w], v + (tok0 + j) * ld + h * d, d);
      ds = expf(s - li) * (dp - di);
    }
    const int jn = min(64, i - j0 + 1);
    for (int jj = 0; jj < jn; ++jj) {
      const float dsj = __shfl(ds, jj, 64);
      const T* kr = k + (tok0 + j0 + jj) * ld + h * d;
#pragma unroll
      for (int c = 0; c < MAXD / 64; ++c)
        if (c * 64 + lane < d) acc[c] += dsj * to_f(kr[c * 64 + lane]);
    }
  }
  T* dqi = dq + (tok0 + i) * ldd + h * d;
#pragma unroll
  for (int c = 0; c < MAXD / 64; ++c)
    if (c * 64 + lane < d) dqi[c * 64 + lane] = from_f<T>(acc[c] * scale);
}

// dv_j = sum_{i>=j} p_ij do_i ;  dk_j = scale * sum_{i>=j} ds_ij q_i
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_simple(int S, int d, const T* __restrict__ q, const T* __restrict__ k,
                                                           const T* __restrict__ v, int64_t ld,
                                                           const T* __restrict__ dout, int64_t ldo,
                                                           const float* __restrict__ lse, const float* __restrict__ delta,
                                                           T* __restrict__ dk, T* __restrict__ dv, int64_t ldd, float scale) {
  __shared__ float ks[4][MAXD];
  __shared__ float vs[4][MAXD];
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int j = blockIdx.x * 4 + w;
  const int h = blockIdx.y, b = blockIdx.z, nh = gridDim.y;
  if (j >= S) return;
  const int64_t tok0 = (int64_t)b * S;
  for (int c = lane; c < d; c += 64) {
    ks[w][c] = to_f(k[(tok0 + j) * ld + h * d + c]) * scale;
    vs[w][c] = to_f(v[(tok0 + j) * ld + h * d + c]);
  }
  __builtin_amdgcn_wave_barrier();
  const float* lrow = lse + ((int64_t)b * nh + h) * S;
  const float* drow = delta + ((int64_t)b * nh + h) * S;
  float acck[MAXD / 64], accv[MAXD / 64];
#pragma unroll
  for (int c = 0; c < MAXD / 64; ++c) acck[c] = accv[c] = 0.f;
  for (int i0 = j; i0 < S; i0 += 64) {
    const int i = i0 + lane;
    float p = 0.f, ds = 0.f;
    if (i < S) {
      const float s = dot_row(ks[w], q + (tok0 + i) * ld + h * d, d);
      const float dp = dot_row(vs[w], dout + (tok0 + i) * ldo + h * d, d);
      p = expf(s - lrow[i]);
      ds = p * (dp - drow[i]);
    }
    const int in = min(64, S - i0);
    for (int ii = 0; ii < in; ++ii) {
      const float pi = __shfl(p, ii, 64);
      const float dsi = __shfl(ds, ii, 64);
      const T* qr = q + (tok0 + i0 + ii) * ld + h * d;
      const T* dor = dout + (tok0 + i0 + ii) * ldo + h * d;
#pragma unroll
      for (int c = 0; c < MAXD / 64; ++c)
        if (c * 64 + lane < d) {
          accv[c] += pi * to_f(dor[c * 64 + lane]);
          acck[c] += dsi * to_f(qr[c * 64 + lane]);
        }
    }
  }
#pragma unroll
  for (int c = 0; c < MAXD / 64; ++c)
    if (c * 64 + lane < d) {
      dk[(tok0 + j) * ldd + h * d + c * 64 + lane] = from_f<T>(acck[c] * scale);
      dv[(tok0 + j) * ldd + h * d + c * 64 + lane] = from_f<T>(accv[c]);
    }
}

template <typename T>
static hipError_t fwd_simple(hipStream_t st, int mb, int S, int nh, int d, const void* q, const void* k, const void* v,
                             int64_t ld, void* o, int64_t ldo, float* lse) {
  dim3 grid((unsigned)cdiv(S, 4), (unsigned)nh, (unsigned)mb), blk(256);
  hipLaunchKernelGGL(attn_fwd_simple<T>, grid, blk, 0, st, S, d, (const T*)q, (const T*)k, (const T*)v, ld, (T*)o, ldo,
                     lse, 1.0f / sqrtf((float)d));
  return hipGetLastError();
}
template <typename T>
static hipError_t bwd_simple(hipStream_t st, int mb, int S, int nh, int d, const void* q, const void* k, const void* v,
                             int64_t ld, const void* o, const void* dout, int64_t ldo, const float* lse, float* delta,
                             void* dq, void* dk, void* dv, int64_t ldd) {
  dim3 grid((unsigned)cdiv(S, 4), (unsigned)nh, (unsigned)mb), blk(256);
  const float scale = 1.0f / sqrtf((float)d);
  hipLaunchKernelGGL(attn_delta_kernel<T>, grid, blk, 0, st, S, d, (const T*)o, (const T*)dout, ldo, delta);
  hipLaunchKernelGGL(attn_bwd_dq_simple<T>, grid, blk, 0, st, S, d, (const T*)q, (const T*)k, (const T*)v, ld,
                     (const T*)dout, ldo, lse, delta, (T*)dq, ldd, scale);
  hipLaunchKernelGGL(attn_bwd_dkv_simple<T>, grid, blk, 0, st, S, d, (const T*)q, (const T*)k, (const T*)v, ld,
                     (const T*)dout, ldo, lse, delta, (T*)dk, (T*)dv, ldd, scale);
  return hipGetLastError();
}

hipError_t attn_fwd_mfma(hipStream_t st, int mb, int S, int nh, int d, const void* q, const void* k, const void* v,
                         int64_t ld, void* o, int64_t ldo, float* lse);
hipError_t attn_bwd_mfma(hipStream_t st, int mb, int S, int nh, int d, const void* q, const void* k, const void* v,
                         int64_t ld, const void* o, const void* dout, int64_t ldo, const float* lse, float* delta,
                         void* dq, void* dk, void* dv, int64_t ldd, const float2* rope);
hipError_t attn_fwd_mfma_f16(hipStream_t st, int mb, int S, int nh, int d, const void* q, const void* k, const void* v,
                             int64_t ld, void* o, int64_t ldo, float* lse);
hipError_t attn_bwd_mfma_f16(hipStream_t st, int mb, int S, int nh, int d, const void* q, const void* k, const void* v,
                             int64_t ld, const void* o, const void* dout, int64_t ldo, const float* lse, float* delta,
                             void* dq, void* dk, void* dv, int64_t ldd, const float2* rope);
bool attn_mfma_supported(DType dt, int S, int d);

int attn_select(DType dt, int S, int d, int force) {
  if (force == ATTN_SIMPLE) return ATTN_SIMPLE;
  return attn_mfma_supported(dt, S, d) ? ATTN_MFMA : ATTN_SIMPLE;
}

hipError_t attn_fwd(hipStream_t st, DType dt, int mb, int S, int nh, int d, const void* q, const void* k,
                    const void* v, int64_t ld, void* o, int64_t ldo, float* lse, int force) {
  if (attn_select(dt, S, d, force) == ATTN_MFMA)
    return dt == F16 ? attn_fwd_mfma_f16(st, mb, S, nh, d, q, k, v, ld, o, ldo, lse)
                     : attn_fwd_mfma(st, mb, S, nh, d, q, k, v, ld, o, ldo, lse);
  return dt == F32    ? fwd_simple<float>(st, mb, S, nh, d, q, k, v, ld, o, ldo, lse)
         : dt == BF16 ? fwd_simple<bf16>(st, mb, S, nh, d, q, k, v, ld, o, ldo, lse)
                      : fwd_simple<f16>(st, mb, S, nh, d, q, k, v, ld, o, ldo, lse);
}
hipError_t attn_bwd(hipStream_t st, DType dt, int mb, int S, int nh, int d, const void* q, const void* k,
                    const void* v, int64_t ld, const void* o, const void* dout, int64_t ldo, const float* lse,
                    float* delta, void* dq, void* dk, void* dv, int64_t ldd, const float2* rope, int force) {
  if (attn_select(dt, S, d, force) == ATTN_MFMA)   // rotation fused into the kernels' stores
    return dt == F16 ? attn_bwd_mfma_f16(st, mb, S, nh, d, q, k, v, ld, o, dout, ldo, lse, delta, dq, dk, dv, ldd, rope)
                     : attn_bwd_mfma(st, mb, S, nh, d, q, k, v, ld, o, dout, ldo, lse, delta, dq, dk, dv, ldd, rope);
  hipError_t e = dt == F32    ? bwd_simple<float>(st, mb, S, nh, d, q, k, v, ld, o, dout, ldo, lse, delta, dq, dk, dv, ldd)
                 : dt == BF16 ? bwd_simple<bf16>(st, mb, S, nh, d, q, k, v, ld, o, dout, ldo, lse, delta, dq, dk, dv, ldd)
                              : bwd_simple<f16>(st, mb, S, nh, d, q, k, v, ld, o, dout, ldo, lse, delta, dq, dk, dv, ldd);
  if (e == hipSuccess && rope) e = rope_apply(st, dt, mb * S, S, nh * d, d, dq, ldd, rope, -1.0f);
  if (e == hipSuccess && rope) e = rope_apply(st, dt, mb * S, S, nh * d, d, dk, ldd, rope, -1.0f);
  return e;
}

}  // namespace zs
