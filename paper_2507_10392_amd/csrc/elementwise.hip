// Bandwidth-bound kernels of the stage step: norms, activations, RoPE, embedding, cross
// entropy, vector-gradient reductions and the fused AdamW.  Statistics and all arithmetic are
// fp32; storage is float or bf16.  Every global access is a 16-byte vector per lane where the
// shape allows it, consecutive lanes touching consecutive vectors.
#include "kernels.h"

namespace zs {

template <typename T> struct VT { typedef typename Vec<T>::type type; };

template <typename T> __device__ __forceinline__ void load_vec(const T* p, float (&out)[Vec<T>::N]) {
  typename Vec<T>::type v = *reinterpret_cast<const typename Vec<T>::type*>(p);
#pragma unroll
  for (int i = 0; i < Vec<T>::N; ++i) out[i] = to_f(v[i]);
}
template <typename T> __device__ __forceinline__ void store_vec(T* p, const float (&in)[Vec<T>::N]) {
  typename Vec<T>::type v;
#pragma unroll
  for (int i = 0; i < Vec<T>::N; ++i) v[i] = from_f<T>(in[i]);
  *reinterpret_cast<typename Vec<T>::type*>(p) = v;
}

// ------------------------------------------------------------------ norm forward
// One wave per row; three passes over a row that stays in cache (mean, variance, output).
template <typename T, int KIND>
__global__ __launch_bounds__(256) void norm_fwd_kernel(int Trows, int H, const T* __restrict__ x,
                                                       const T* __restrict__ g, const T* __restrict__ b, float eps,
                                                       T* __restrict__ n, float* __restrict__ rstd,
                                                       float* __restrict__ mean) {
  constexpr int V = Vec<T>::N;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= Trows) return;
  const T* xr = x + (int64_t)row * H;
  float mu = 0.f;
  if (KIND == 0) {
    float s = 0.f;
    for (int c = lane * V; c < H; c += 64 * V) {
      float a[V];
      load_vec(xr + c, a);
#pragma unroll
      for (int i = 0; i < V; ++i) s += a[i];
    }
    mu = wave_sum(s) / (float)H;
  }
  float s2 = 0.f;
  for (int c = lane * V; c < H; c += 64 * V) {
    float a[V];
    load_vec(xr + c, a);
#pragma unroll
    for (int i = 0; i < V; ++i) s2 += (a[i] - mu) * (a[i] - mu);
  }
  const float r = 1.0f / sqrtf(wave_sum(s2) / (float)H + eps);
  if (lane == 0) {
    rstd[row] = r;
    if (KIND == 0) mean[row] = mu;
  }
  T* nr = n + (int64_t)row * H;
  for (int c = lane * V; c < H; c += 64 * V) {
    float a[V], gg[V], bb[V], o[V];
    load_vec(xr + c, a);
    load_vec(g + c, gg);
    if (KIND == 0) load_vec(b + c, bb);
#pragma unroll
    for (int i = 0; i < V; ++i) o[i] = (a[i] - mu) * r * gg[i] + (KIND == 0 ? bb[i] : 0.f);
    store_vec(nr + c, o);
  }
}

// Same arithmetic with the row kept in registers (one global read): H = 64 lanes x V x J exactly.  The
// element -> lane assignment and the order of every sum equal the kernel above, so the results are identical.
template <typename T, int KIND, int J>
__global__ __launch_bounds__(256) void norm_fwd_reg_kernel(int Trows, const T* __restrict__ x, const T* __restrict__ g,
                                                           const T* __restrict__ b, float eps, T* __restrict__ n,
                                                           float* __restrict__ rstd, float* __restrict__ mean) {
  constexpr int V = Vec<T>::N, H = 64 * V * J;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= Trows) return;
  const T* xr = x + (int64_t)row * H;
  float a[J][V];
#pragma unroll
  for (int j = 0; j < J; ++j) load_vec(xr + (j * 64 + lane) * V, a[j]);
  float mu = 0.f;
  if (KIND == 0) {
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < J; ++j)
#pragma unroll
      for (int i = 0; i < V; ++i) s += a[j][i];
    mu = wave_sum(s) / (float)H;
  }
  float s2 = 0.f;
#pragma unroll
  for (int j = 0; j < J; ++j)
#pragma unroll
    for (int i = 0; i < V; ++i) s2 += (a[j][i] - mu) * (a[j][i] - mu);
  const float r = 1.0f / sqrtf(wave_sum(s2) / (float)H + eps);
  if (lane == 0) {
    rstd[row] = r;
    if (KIND == 0) mean[row] = mu;
  }
  T* nr = n + (int64_t)row * H;
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int c = (j * 64 + lane) * V;
    float gg[V], bb[V], o[V];
    load_vec(g + c, gg);
    if (KIND == 0) load_vec(b + c, bb);
#pragma unroll
    for (int i = 0; i < V; ++i) o[i] = (a[j][i] - mu) * r * gg[i] + (KIND == 0 ? bb[i] : 0.f);
    store_vec(nr + c, o);
  }
}

// J (row = 64 x V x J elements) for which the register-resident norm kernels are instantiated, else 0.
static int reg_chunks(DType dt, int H) {
  const int per = 64 * (dt == F32 ? 4 : 8);   // both 16-bit types move 8 elements per access
  if (H % per) return 0;
  const int J = H / per;
  return (J == 1 || J == 2 || J == 4 || J == 8 || J == 10) ? J : 0;
}

hipError_t norm_fwd(hipStream_t st, DType dt, int kind, int T, int H, const void* x, const void* g, const void* b,
                    float eps, void* n, float* rstd, float* mean) {
  dim3 grid((unsigned)cdiv(T, 4)), blk(256);
  const int J = reg_chunks(dt, H);
#define LR(TT, KK, JJ) \
  hipLaunchKernelGGL((norm_fwd_reg_kernel<TT, KK, JJ>), grid, blk, 0, st, T, (const TT*)x, (const TT*)g, (const TT*)b, eps, (TT*)n, rstd, mean)
#define LJ(TT, KK) \
  switch (J) { case 1: LR(TT, KK, 1); break; case 2: LR(TT, KK, 2); break; case 4: LR(TT, KK, 4); break; \
               case 8: LR(TT, KK, 8); break; default: LR(TT, KK, 10); break; }
#define L(TT, KK) \
  hipLaunchKernelGGL((norm_fwd_kernel<TT, KK>), grid, blk, 0, st, T, H, (const TT*)x, (const TT*)g, (const TT*)b, eps, (TT*)n, rstd, mean)
  if (J) {
    if (dt == F32) { if (kind == 0) { LJ(float, 0) } else { LJ(float, 1) } }
    else if (dt == BF16) { if (kind == 0) { LJ(bf16, 0) } else { LJ(bf16, 1) } }
    else { if (kind == 0) { LJ(f16, 0) } else { LJ(f16, 1) } }
  } else {
    if (dt == F32) { if (kind == 0) L(float, 0); else L(float, 1); }
    else if (dt == BF16) { if (kind == 0) L(bf16, 0); else L(bf16, 1); }
    else { if (kind == 0) L(f16, 0); else L(f16, 1); }
  }
#undef L
#undef LJ
#undef LR
  return hipGetLastError();
}

// ------------------------------------------------------------------ norm backward (dx only)
// u = dn*g; dx = r*(u - mean(u) [LN] - xhat*mean(u*xhat)) + dres
template <typename T, int KIND>
__global__ __launch_bounds__(256) void norm_bwd_kernel(int Trows, int H, const T* __restrict__ dn,
                                                       const T* __restrict__ x, const T* __restrict__ g,
                                                       const float* __restrict__ rstd, const float* __restrict__ mean,
                                                       const T* dres, T* dx) {
  constexpr int V = Vec<T>::N;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= Trows) return;
  const float r = rstd[row];
  const float mu = (KIND == 0) ? mean[row] : 0.f;
  const T* xr = x + (int64_t)row * H;
  const T* dr = dn + (int64_t)row * H;
  float su = 0.f, sux = 0.f;
  for (int c = lane * V; c < H; c += 64 * V) {
    float a[V], d[V], gg[V];
    load_vec(xr + c, a);
    load_vec(dr + c, d);
    load_vec(g + c, gg);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      const float u = d[i] * gg[i];
      su += u;
      sux += u * (a[i] - mu) * r;
    }
  }
  const float mu_u = (KIND == 0) ? wave_sum(su) / (float)H : 0.f;
  const float mu_ux = wave_sum(sux) / (float)H;
  for (int c = lane * V; c < H; c += 64 * V) {
    float a[V], d[V], gg[V], o[V], rs[V];
    load_vec(xr + c, a);
    load_vec(dr + c, d);
    load_vec(g + c, gg);
    if (dres) load_vec(dres + (int64_t)row * H + c, rs);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      const float u = d[i] * gg[i];
      o[i] = r * (u - mu_u - (a[i] - mu) * r * mu_ux) + (dres ? rs[i] : 0.f);
    }
    store_vec(dx + (int64_t)row * H + c, o);
  }
}

// ------------------------------------------------------------------ norm backward, row in registers
// dx as norm_bwd_kernel with each row read once and kept in registers as stored (H = 64 x V x J); same
// element -> lane assignment and summation order, hence identical results.
template <typename T, int KIND, int J>
__global__ __launch_bounds__(256) void norm_bwd_reg_kernel(int Trows, const T* __restrict__ dn, const T* __restrict__ x,
                                                           const T* __restrict__ g, const float* __restrict__ rstd,
                                                           const float* __restrict__ mean, const T* dres, T* dx) {
  constexpr int V = Vec<T>::N, H = 64 * V * J;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= Trows) return;
  const float r = rstd[row];
  const float mu = (KIND == 0) ? mean[row] : 0.f;
  const int64_t off = (int64_t)row * H;
  typename Vec<T>::type xv[J], dv[J];
  float su = 0.f, sux = 0.f;
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int c = (j * 64 + lane) * V;
    xv[j] = *reinterpret_cast<const typename Vec<T>::type*>(x + off + c);
    dv[j] = *reinterpret_cast<const typename Vec<T>::type*>(dn + off + c);
    float gg[V];
    load_vec(g + c, gg);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      const float u = to_f(dv[j][i]) * gg[i];
      su += u;
      sux += u * (to_f(xv[j][i]) - mu) * r;
    }
  }
  const float mu_u = (KIND == 0) ? wave_sum(su) / (float)H : 0.f;
  const float mu_ux = wave_sum(sux) / (float)H;
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int c = (j * 64 + lane) * V;
    float o[V], rs[V], gg[V];
    load_vec(g + c, gg);
    if (dres) load_vec(dres + off + c, rs);
#pragma unroll
    for (int i = 0; i < V; ++i) {
      const float u = to_f(dv[j][i]) * gg[i];
      o[i] = r * (u - mu_u - (to_f(xv[j][i]) - mu) * r * mu_ux) + (dres ? rs[i] : 0.f);
    }
    store_vec(dx + off + c, o);
  }
}

hipError_t norm_bwd(hipStream_t st, DType dt, int kind, int T, int H, const void* dn, const void* x, const void* g,
                    const float* rstd, const float* mean, const void* dres, void* dx) {
  dim3 grid((unsigned)cdiv(T, 4)), blk(256);
  const int J = reg_chunks(dt, H);
#define LR(TT, KK, JJ) \
  hipLaunchKernelGGL((norm_bwd_reg_kernel<TT, KK, JJ>), grid, blk, 0, st, T, (const TT*)dn, (const TT*)x, (const TT*)g, rstd, mean, (const TT*)dres, (TT*)dx)
#define LJ(TT, KK) \
  switch (J) { case 1: LR(TT, KK, 1); break; case 2: LR(TT, KK, 2); break; case 4: LR(TT, KK, 4); break; \
               case 8: LR(TT, KK, 8); break; default: LR(TT, KK, 10); break; }
#define L(TT, KK) \
  hipLaunchKernelGGL((norm_bwd_kernel<TT, KK>), grid, blk, 0, st, T, H, (const TT*)dn, (const TT*)x, (const TT*)g, rstd, mean, (const TT*)dres, (TT*)dx)
  if (J) {
    if (dt == F32) { if (kind == 0) { LJ(float, 0) } else { LJ(float, 1) } }
    else if (dt == BF16) { if (kind == 0) { LJ(bf16, 0) } else { LJ(bf16, 1) } }
    else { if (kind == 0) { LJ(f16, 0) } else { LJ(f16, 1) } }
  } else {
    if (dt == F32) { if (kind == 0) L(float, 0); else L(float, 1); }
    else if (dt == BF16) { if (kind == 0) L(bf16, 0); else L(bf16, 1); }
    else { if (kind == 0) L(f16, 0); else L(f16, 1); }
  }
#undef L
#undef LJ
#undef LR
  return hipGetLastError();
}

// ------------------------------------------------------------------ column partial sums
// grid (column chunks of 64*V, nblk).  A workgroup is 64 column threads (V columns each) x 4 row groups:
// row group q walks rows r0+q, r0+q+4, ... of the block, four rows in flight per thread, and the four
// groups' sums are added in the order 0..3 through LDS, so the result does not depend on timing.
template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(int Trows, int N, const T* __restrict__ a, int64_t lda,
                                                     const T* __restrict__ x, int64_t ldx,
                                                     const float* __restrict__ rstd, const float* __restrict__ mean,
                                                     float* __restrict__ part, int rows_per_blk) {
  constexpr int V = Vec<T>::N;
  __shared__ float red[3][64][V];
  const int ct = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int col = (blockIdx.x * 64 + ct) * V;
  const bool live = col < N;
  const int r0 = blockIdx.y * rows_per_blk;
  const int r1 = min(Trows, r0 + rows_per_blk);
  float acc[V];
#pragma unroll
  for (int i = 0; i < V; ++i) acc[i] = 0.f;
  if (live) {
    for (int t0 = r0 + q; t0 < r1; t0 += 16) {
      float av[4][V], xv[4][V];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int t = t0 + 4 * u;
        if (t < r1) {
          load_vec(a + (int64_t)t * lda + col, av[u]);
          if (x) load_vec(x + (int64_t)t * ldx + col, xv[u]);
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int t = t0 + 4 * u;
        if (t < r1) {
          if (x) {
            const float r = rstd[t];
            const float mu = mean ? mean[t] : 0.f;
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] += av[u][i] * ((xv[u][i] - mu) * r);
          } else {
#pragma unroll
            for (int i = 0; i < V; ++i) acc[i] += av[u][i];
          }
        }
      }
    }
  }
  if (q > 0) {
#pragma unroll
    for (int i = 0; i < V; ++i) red[q - 1][ct][i] = acc[i];
  }
  __syncthreads();
  if (q == 0 && live) {
    float* p = part + (int64_t)blockIdx.y * N + col;
#pragma unroll
    for (int i = 0; i < V; ++i) p[i] = ((acc[i] + red[0][ct][i]) + red[1][ct][i]) + red[2][ct][i];
  }
}

hipError_t colsum_partial(hipStream_t st, DType dt, int T, int N, const void* a, int64_t lda, const void* x,
                          int64_t ldx, const float* rstd, const float* mean, float* part, int nblk) {
  const int rows_per_blk = (int)cdiv(T, nblk);
  const int V = dt == F32 ? 4 : 8;
  dim3 grid((unsigned)cdiv(N, 64 * V), (unsigned)nblk), blk(256);
  if (dt == F32)
    hipLaunchKernelGGL(colsum_kernel<float>, grid, blk, 0, st, T, N, (const float*)a, lda, (const float*)x, ldx, rstd, mean, part, rows_per_blk);
  else if (dt == BF16)
    hipLaunchKernelGGL(colsum_kernel<bf16>, grid, blk, 0, st, T, N, (const bf16*)a, lda, (const bf16*)x, ldx, rstd, mean, part, rows_per_blk);
  else
    hipLaunchKernelGGL(colsum_kernel<f16>, grid, blk, 0, st, T, N, (const f16*)a, lda, (const f16*)x, ldx, rstd, mean, part, rows_per_blk);
  return hipGetLastError();
}

// ------------------------------------------------------------------ norm backward + partial sums, row in registers
// norm_bwd_reg_kernel and the two colsum_kernel passes over the same rows in one kernel: dn and x are read once.
// One workgroup per row block (the blocks of colsum_partial); wave q walks rows r0+q, r0+q+4, ... of the block,
// computes dx of each row as norm_bwd_reg_kernel does and keeps the running column sums of dn*xhat (and dn) of
// its rows in registers; the four waves' sums are then added in the order 0..3 through LDS.  That is colsum_kernel's
// order of additions per column, so the partial sums do not depend on which of the two routes ran.
template <typename T, int KIND, int J>
__global__ __launch_bounds__(256) void norm_bwd_partials_reg_kernel(int Trows, const T* __restrict__ dn, const T* __restrict__ x,
                                                                    const T* __restrict__ g, const float* __restrict__ rstd,
                                                                    const float* __restrict__ mean, const T* dres, T* dx,
                                                                    float* __restrict__ part_g, float* __restrict__ part_b,
                                                                    int rows_per_blk) {
  constexpr int V = Vec<T>::N, H = 64 * V * J;
  extern __shared__ __align__(16) float red[];   // [3][H]: the sums of waves 1..3, used for part_g and then for part_b
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int r0 = blockIdx.x * rows_per_blk;
  const int r1 = min(Trows, r0 + rows_per_blk);
  float pg[J][V], pb[KIND == 0 ? J : 1][V];
#pragma unroll
  for (int j = 0; j < J; ++j)
#pragma unroll
    for (int i = 0; i < V; ++i) { pg[j][i] = 0.f; if (KIND == 0) pb[j][i] = 0.f; }
  for (int row = r0 + q; row < r1; row += 4) {
    const float r = rstd[row];
    const float mu = (KIND == 0) ? mean[row] : 0.f;
    const int64_t off = (int64_t)row * H;
    typename Vec<T>::type xv[J], dv[J], rv[J];
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const int c = (j * 64 + lane) * V;
      xv[j] = *reinterpret_cast<const typename Vec<T>::type*>(x + off + c);
      dv[j] = *reinterpret_cast<const typename Vec<T>::type*>(dn + off + c);
      if (dres) rv[j] = *reinterpret_cast<const typename Vec<T>::type*>(dres + off + c);
    }
    float su = 0.f, sux = 0.f;
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const int c = (j * 64 + lane) * V;
      float gg[V];
      load_vec(g + c, gg);
#pragma unroll
      for (int i = 0; i < V; ++i) {
        const float d = to_f(dv[j][i]), xx = to_f(xv[j][i]);
        const float u = d * gg[i];
        su += u;
        sux += u * (xx - mu) * r;
        pg[j][i] += d * ((xx - mu) * r);
        if (KIND == 0) pb[j][i] += d;
      }
    }
    const float mu_u = (KIND == 0) ? wave_sum(su) / (float)H : 0.f;
    const float mu_ux = wave_sum(sux) / (float)H;
#pragma unroll
    for (int j = 0; j < J; ++j) {
      const int c = (j * 64 + lane) * V;
      float o[V], gg[V];
      load_vec(g + c, gg);
#pragma unroll
      for (int i = 0; i < V; ++i) {
        const float u = to_f(dv[j][i]) * gg[i];
        o[i] = r * (u - mu_u - (to_f(xv[j][i]) - mu) * r * mu_ux) + (dres ? to_f(rv[j][i]) : 0.f);
      }
      store_vec(dx + off + c, o);
    }
  }
  // cross-wave sums in the order 0..3, first of dn*xhat, then (LayerNorm) of dn
#pragma unroll
  for (int pass = 0; pass < (KIND == 0 ? 2 : 1); ++pass) {
    if (pass) __syncthreads();
    // LDS layout [wave][j][quad of 4 columns][lane]: consecutive lanes 16 bytes apart, no bank conflicts
    constexpr int Q4 = V / 4;
    f32x4* red4 = reinterpret_cast<f32x4*>(red);
    if (q > 0) {
#pragma unroll
      for (int j = 0; j < J; ++j)
#pragma unroll
        for (int h = 0; h < Q4; ++h) {
          f32x4 t;
#pragma unroll
          for (int e = 0; e < 4; ++e) t[e] = pass ? pb[j][4 * h + e] : pg[j][4 * h + e];
          red4[(((q - 1) * J + j) * Q4 + h) * 64 + lane] = t;
        }
    }
    __syncthreads();
    if (q == 0) {
      float* p = (pass ? part_b : part_g) + (int64_t)blockIdx.x * H;
#pragma unroll
      for (int j = 0; j < J; ++j) {
        const int c = (j * 64 + lane) * V;
#pragma unroll
        for (int h = 0; h < Q4; ++h) {
          const f32x4 r1 = red4[((0 * J + j) * Q4 + h) * 64 + lane], r2 = red4[((1 * J + j) * Q4 + h) * 64 + lane],
                      r3 = red4[((2 * J + j) * Q4 + h) * 64 + lane];
          f32x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (((pass ? pb[j][4 * h + e] : pg[j][4 * h + e]) + r1[e]) + r2[e]) + r3[e];
          *reinterpret_cast<f32x4*>(p + c + 4 * h) = o;
        }
      }
    }
  }
}

hipError_t norm_bwd_partials(hipStream_t st, DType dt, int kind, int T, int H, const void* dn, const void* x, const void* g,
                             const float* rstd, const float* mean, const void* dres, void* dx, float* part_g,
                             float* part_b, int nblk) {
  const int J = reg_chunks(dt, H);
  if (J && nblk >= 1 && part_g && (kind != 0 || part_b)) {   // one pass over the rows
    const int rows_per_blk = (int)cdiv(T, nblk);
    dim3 grid((unsigned)nblk), blk(256);
    const size_t smem = 3 * (size_t)H * sizeof(float);
#define LR(TT, KK, JJ) \
  hipLaunchKernelGGL((norm_bwd_partials_reg_kernel<TT, KK, JJ>), grid, blk, smem, st, T, (const TT*)dn, (const TT*)x, (const TT*)g, rstd, mean, (const TT*)dres, (TT*)dx, part_g, part_b, rows_per_blk)
#define LJ(TT, KK) \
  switch (J) { case 1: LR(TT, KK, 1); break; case 2: LR(TT, KK, 2); break; case 4: LR(TT, KK, 4); break; \
               case 8: LR(TT, KK, 8); break; default: LR(TT, KK, 10); break; }
    if (dt == F32) { if (kind == 0) { LJ(float, 0) } else { LJ(float, 1) } }
    else if (dt == BF16) { if (kind == 0) { LJ(bf16, 0) } else { LJ(bf16, 1) } }
    else { if (kind == 0) { LJ(f16, 0) } else { LJ(f16, 1) } }
#undef LJ
#undef LR
    return hipGetLastError();
  }
  hipError_t e = colsum_partial(st, dt, T, H, dn, H, x, H, rstd, kind == 0 ? mean : nullptr, part_g, nblk);
  if (e == hipSuccess && kind == 0) e = colsum_partial(st, dt, T, H, dn, H, nullptr, H, nullptr, nullptr, part_b, nblk);
  if (e == hipSuccess) e = norm_bwd(st, dt, kind, T, H, dn, x, g, rstd, mean, dres, dx);
  return e;
}

// dst[c] += sum over the blocks, formed as four interleaved running sums (blocks b, b+4, ...) that are
// added in the order 0..3 at the end: a fixed order, with four loads in flight per thread.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const ReduceJob* __restrict__ jobs) {
  const ReduceJob j = jobs[blockIdx.x];
  const int c = blockIdx.y * 256 + threadIdx.x;
  if (c >= j.width) return;
  float s[4] = {0.f, 0.f, 0.f, 0.f};
  const float* p = j.part + c;
  int b = 0;
  for (; b + 4 <= j.nblk; b += 4) {
#pragma unroll
    for (int u = 0; u < 4; ++u) s[u] += p[(int64_t)(b + u) * j.width];
  }
  for (int u = 0; b < j.nblk; ++b, ++u) s[u] += p[(int64_t)b * j.width];
  j.dst[c] += ((s[0] + s[1]) + s[2]) + s[3];
}

hipError_t reduce_partials(hipStream_t st, const ReduceJob* jobs_dev, int njobs, int max_width) {
  if (njobs == 0) return hipSuccess;
  dim3 grid((unsigned)njobs, (unsigned)cdiv(max_width, 256)), blk(256);
  hipLaunchKernelGGL(reduce_partials_kernel, grid, blk, 0, st, jobs_dev);
  return hipGetLastError();
}

// ------------------------------------------------------------------ RoPE
__global__ void rope_table_kernel(int S, int d, double base, float2* table) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int half = d / 2;
  if (idx >= S * half) return;
  const int s = idx / half, i = idx % half;
  const double theta = (double)s * pow(base, -2.0 * (double)i / (double)d);
  table[idx] = make_float2((float)cos(theta), (float)sin(theta));
}
hipError_t rope_table(hipStream_t st, int S, int d, float base, float2* table) {
  const int n = S * (d / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, st, S, d, (double)base, table);
  return hipGetLastError();
}

template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(int Trows, int S, int ncols, int d, T* a, int64_t ld,
                                                   const float2* __restrict__ table, float sign) {
  constexpr int V = Vec<T>::N;
  const int vec_per_row = ncols / V;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)Trows * vec_per_row) return;
  const int t = (int)(idx / vec_per_row);
  const int c = (int)(idx % vec_per_row) * V;
  const int pos = t % S;
  T* p = a + (int64_t)t * ld + c;
  float u[V], o[V];
  load_vec(p, u);
  const int i0 = (c % d) / 2;
#pragma unroll
  for (int i = 0; i < V / 2; ++i) {
    const float2 cs = table[pos * (d / 2) + i0 + i];
    const float sn = sign * cs.y;
    o[2 * i] = u[2 * i] * cs.x - u[2 * i + 1] * sn;
    o[2 * i + 1] = u[2 * i] * sn + u[2 * i + 1] * cs.x;
  }
  store_vec(p, o);
}
hipError_t rope_apply(hipStream_t st, DType dt, int T, int S, int ncols, int d, void* a, int64_t ld,
                      const float2* table, float sign) {
  const int V = dt == F32 ? 4 : 8;
  const int64_t n = (int64_t)T * (ncols / V);
  dim3 grid((unsigned)cdiv(n, 256)), blk(256);
  if (dt == F32) hipLaunchKernelGGL(rope_kernel<float>, grid, blk, 0, st, T, S, ncols, d, (float*)a, ld, table, sign);
  else if (dt == BF16) hipLaunchKernelGGL(rope_kernel<bf16>, grid, blk, 0, st, T, S, ncols, d, (bf16*)a, ld, table, sign);
  else hipLaunchKernelGGL(rope_kernel<f16>, grid, blk, 0, st, T, S, ncols, d, (f16*)a, ld, table, sign);
  return hipGetLastError();
}

// ------------------------------------------------------------------ activations
// GELU(z) = z Phi(z) with Phi the normal distribution function (the erf form) and its derivative Phi(z) + z phi(z).
// erf comes from the rational approximation 7.1.26 of Abramowitz and Stegun, |error| <= 1.5e-7, i.e. fp32 rounding level:
// erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1 / (1 + p x), x >= 0.  With x = |z| / sqrt(2) its exponential is
// exp(-z^2 / 2), the one the density phi needs as well, so value and derivative cost one hardware exp2 and one hardware
// reciprocal instead of erff and expf (these kernels were bound by that arithmetic, not by memory).
__device__ __forceinline__ void gelu_parts(float z, float& Phi, float& phi) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * x * x);
  const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * x);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  Phi = 0.5f * (1.0f + copysignf(1.0f - poly * e, z));
  phi = 0.39894228040143268f * e;
}
__device__ __forceinline__ float gelu_f(float z) {
  float Phi, phi;
  gelu_parts(z, Phi, phi);
  return z * Phi;
}
__device__ __forceinline__ float gelu_df(float z) {
  float Phi, phi;
  gelu_parts(z, Phi, phi);
  return Phi + z * phi;
}

template <typename T, int MODE>  // 0: a = gelu(z); 1: dz = da * gelu'(z)
__global__ __launch_bounds__(256) void gelu_kernel(int64_t nvec, const T* __restrict__ z, const T* __restrict__ da,
                                                   T* __restrict__ out) {
  constexpr int V = Vec<T>::N;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= nvec) return;
  float zz[V], o[V], d[V];
  load_vec(z + i * V, zz);
  if (MODE == 1) load_vec(da + i * V, d);
#pragma unroll
  for (int k = 0; k < V; ++k) o[k] = MODE == 0 ? gelu_f(zz[k]) : d[k] * gelu_df(zz[k]);
  store_vec(out + i * V, o);
}
hipError_t gelu_fwd(hipStream_t st, DType dt, int64_t n, const void* z, void* a) {
  const int V = dt == F32 ? 4 : 8;
  dim3 grid((unsigned)cdiv(n / V, 256)), blk(256);
  if (dt == F32) hipLaunchKernelGGL((gelu_kernel<float, 0>), grid, blk, 0, st, n / V, (const float*)z, (const float*)nullptr, (float*)a);
  else if (dt == BF16) hipLaunchKernelGGL((gelu_kernel<bf16, 0>), grid, blk, 0, st, n / V, (const bf16*)z, (const bf16*)nullptr, (bf16*)a);
  else hipLaunchKernelGGL((gelu_kernel<f16, 0>), grid, blk, 0, st, n / V, (const f16*)z, (const f16*)nullptr, (f16*)a);
  return hipGetLastError();
}
hipError_t gelu_bwd(hipStream_t st, DType dt, int64_t n, const void* z, const void* da, void* dz) {
  const int V = dt == F32 ? 4 : 8;
  dim3 grid((unsigned)cdiv(n / V, 256)), blk(256);
  if (dt == F32) hipLaunchKernelGGL((gelu_kernel<float, 1>), grid, blk, 0, st, n / V, (const float*)z, (const float*)da, (float*)dz);
  else if (dt == BF16) hipLaunchKernelGGL((gelu_kernel<bf16, 1>), grid, blk, 0, st, n / V, (const bf16*)z, (const bf16*)da, (bf16*)dz);
  else hipLaunchKernelGGL((gelu_kernel<f16, 1>), grid, blk, 0, st, n / V, (const f16*)z, (const f16*)da, (f16*)dz);
  return hipGetLastError();
}

template <typename T, int MODE>  // 0: a = silu(g)*u ; 1: (dg, du) from da
__global__ __launch_bounds__(256) void swiglu_kernel(int Trows, int F, const T* gu, const T* __restrict__ da, T* out) {
  constexpr int V = Vec<T>::N;
  const int vec_per_row = F / V;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)Trows * vec_per_row) return;
  const int t = (int)(idx / vec_per_row);
  const int c = (int)(idx % vec_per_row) * V;
  float g[V], u[V];
  load_vec(gu + (int64_t)t * 2 * F + c, g);
  load_vec(gu + (int64_t)t * 2 * F + F + c, u);
  if (MODE == 0) {
    float o[V];
#pragma unroll
    for (int k = 0; k < V; ++k) o[k] = glu_f(g[k], u[k]);
    store_vec(out + (int64_t)t * F + c, o);
  } else {
    float d[V], dg[V], du[V];
    load_vec(da + (int64_t)t * F + c, d);
#pragma unroll
    for (int k = 0; k < V; ++k) glu_df(d[k], g[k], u[k], dg[k], du[k]);
    store_vec(out + (int64_t)t * 2 * F + c, dg);
    store_vec(out + (int64_t)t * 2 * F + F + c, du);
  }
}
hipError_t swiglu_fwd(hipStream_t st, DType dt, int T, int F, const void* gu, void* a) {
  const int V = dt == F32 ? 4 : 8;
  dim3 grid((unsigned)cdiv((int64_t)T * (F / V), 256)), blk(256);
  if (dt == F32) hipLaunchKernelGGL((swiglu_kernel<float, 0>), grid, blk, 0, st, T, F, (const float*)gu, (const float*)nullptr, (float*)a);
  else if (dt == BF16) hipLaunchKernelGGL((swiglu_kernel<bf16, 0>), grid, blk, 0, st, T, F, (const bf16*)gu, (const bf16*)nullptr, (bf16*)a);
  else hipLaunchKernelGGL((swiglu_kernel<f16, 0>), grid, blk, 0, st, T, F, (const f16*)gu, (const f16*)nullptr, (f16*)a);
  return hipGetLastError();
}
hipError_t swiglu_bwd(hipStream_t st, DType dt, int T, int F, const void* gu, const void* da, void* dgu) {
  const int V = dt == F32 ? 4 : 8;
  dim3 grid((unsigned)cdiv((int64_t)T * (F / V), 256)), blk(256);
  if (dt == F32) hipLaunchKernelGGL((swiglu_kernel<float, 1>), grid, blk, 0, st, T, F, (const float*)gu, (const float*)da, (float*)dgu);
  else if (dt == BF16) hipLaunchKernelGGL((swiglu_kernel<bf16, 1>), grid, blk, 0, st, T, F, (const bf16*)gu, (const bf16*)da, (bf16*)dgu);
  else hipLaunchKernelGGL((swiglu_kernel<f16, 1>), grid, blk, 0, st, T, F, (const f16*)gu, (const f16*)da, (f16*)dgu);
  return hipGetLastError();
}

// ------------------------------------------------------------------ embedding
template <typename T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(int H, int V, const int32_t* __restrict__ ids,
                                                        const T* __restrict__ E, T* __restrict__ x) {
  constexpr int VN = Vec<T>::N;
  typedef typename Vec<T>::type vec_t;
  const int t = blockIdx.x;
  const int id = ids[t];
  const bool ok = id >= 0 && id < V;
  for (int c = threadIdx.x * VN; c < H; c += 256 * VN) {
    vec_t v;
    if (ok) v = *reinterpret_cast<const vec_t*>(E + (int64_t)id * H + c);   // bit-exact row copy
    else {
#pragma unroll
      for (int i = 0; i < VN; ++i) v[i] = from_f<T>(0.f);
    }
    *reinterpret_cast<vec_t*>(x + (int64_t)t * H + c) = v;
  }
}
hipError_t embed_fwd(hipStream_t st, DType dt, int T, int H, int V, const int32_t* ids, const void* E, void* x) {
  if (dt == F32) hipLaunchKernelGGL(embed_fwd_kernel<float>, dim3(T), dim3(256), 0, st, H, V, ids, (const float*)E, (float*)x);
  else if (dt == BF16) hipLaunchKernelGGL(embed_fwd_kernel<bf16>, dim3(T), dim3(256), 0, st, H, V, ids, (const bf16*)E, (bf16*)x);
  else hipLaunchKernelGGL(embed_fwd_kernel<f16>, dim3(T), dim3(256), 0, st, H, V, ids, (const f16*)E, (f16*)x);
  return hipGetLastError();
}

// One workgroup per token.  The workgroup of the FIRST token carrying an id adds the rows of
// every token with that id, in increasing token order, to dE[id]; the others exit.  A row of dE
// has one owner workgroup and a column one owner thread, so no atomics are needed and the
// result does not depend on scheduling.
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_kernel(int Trows, int H, int V, const int32_t* __restrict__ ids,
                                                        const T* __restrict__ dx, float* __restrict__ dE) {
  __shared__ int flags[256];
  const int t = blockIdx.x;
  const int id = ids[t];
  if (id < 0 || id >= V) return;
  int earlier = 0;
  for (int u = threadIdx.x; u < t; u += 256) earlier |= (ids[u] == id);
  if (__syncthreads_or(earlier)) return;
  for (int base = t; base < Trows; base += 256) {
    const int u = base + threadIdx.x;
    const int match = (u < Trows) && (ids[u] == id);
    flags[threadIdx.x] = match;
    if (__syncthreads_or(match)) {
      for (int j = 0; j < 256; ++j) {
        if (!flags[j]) continue;
        for (int c = threadIdx.x; c < H; c += 256) dE[(int64_t)id * H + c] += to_f(dx[(int64_t)(base + j) * H + c]);
      }
    }
    __syncthreads();
  }
}
hipError_t embed_bwd(hipStream_t st, DType dt, int T, int H, int V, const int32_t* ids, const void* dx, float* dE) {
  if (dt == F32) hipLaunchKernelGGL(embed_bwd_kernel<float>, dim3(T), dim3(256), 0, st, T, H, V, ids, (const float*)dx, dE);
  else if (dt == BF16) hipLaunchKernelGGL(embed_bwd_kernel<bf16>, dim3(T), dim3(256), 0, st, T, H, V, ids, (const bf16*)dx, dE);
  else hipLaunchKernelGGL(embed_bwd_kernel<f16>, dim3(T), dim3(256), 0, st, T, H, V, ids, (const f16*)dx, dE);
  return hipGetLastError();
}

// ------------------------------------------------------------------ cross entropy
// One workgroup per row, two passes over the row (maximum, then sum of exponentials; the second pass hits in L2).
// VEC: 16-byte accesses (V and ldz multiples of the vector width, z 16-byte aligned), else element by element.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void ce_fwd_kernel(int V, const T* __restrict__ z, int64_t ldz,
                                                     const int32_t* __restrict__ targets, float* __restrict__ lse,
                                                     float* __restrict__ rowloss) {
  constexpr int VN = Vec<T>::N;
  __shared__ float red[4];
  const int t = blockIdx.x;
  const T* zr = z + (int64_t)t * ldz;
  float mx = -INFINITY;
  if (VEC) {
    for (int c = threadIdx.x * VN; c < V; c += 256 * VN) {
      float a[VN];
      load_vec(zr + c, a);
#pragma unroll
      for (int i = 0; i < VN; ++i) mx = fmaxf(mx, a[i]);
    }
  } else {
    for (int c = threadIdx.x; c < V; c += 256) mx = fmaxf(mx, to_f(zr[c]));
  }
  mx = wave_max(mx);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float s = 0.f;
  if (VEC) {
    for (int c = threadIdx.x * VN; c < V; c += 256 * VN) {
      float a[VN];
      load_vec(zr + c, a);
#pragma unroll
      for (int i = 0; i < VN; ++i) s += expf(a[i] - mx);
    }
  } else {
    for (int c = threadIdx.x; c < V; c += 256) s += expf(to_f(zr[c]) - mx);
  }
  s = block_sum<4>(s, red);
  if (threadIdx.x == 0) {
    const float l = mx + logf(s);
    const int tg = targets[t];
    lse[t] = l;
    rowloss[t] = (tg >= 0 && tg < V) ? l - to_f(zr[tg]) : 0.f;
  }
}
__global__ __launch_bounds__(256) void mean_kernel(int n, const float* __restrict__ v, float* __restrict__ out) {
  __shared__ float red[4];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) s += v[i];
  s = block_sum<4>(s, red);
  if (threadIdx.x == 0) *out = s / (float)n;
}
hipError_t ce_fwd(hipStream_t st, DType dt, int T, int V, const void* z, int64_t ldz, const int32_t* targets,
                  float* lse, float* rowloss, float* loss) {
  const int VN = dt == F32 ? 4 : 8;
  const bool vec = V % VN == 0 && ldz % VN == 0 && ((uintptr_t)z & 15) == 0;
#define CE_FWD(TT) \
  if (vec) hipLaunchKernelGGL((ce_fwd_kernel<TT, true>), dim3(T), dim3(256), 0, st, V, (const TT*)z, ldz, targets, lse, rowloss); \
  else hipLaunchKernelGGL((ce_fwd_kernel<TT, false>), dim3(T), dim3(256), 0, st, V, (const TT*)z, ldz, targets, lse, rowloss)
  if (dt == F32) { CE_FWD(float); } else if (dt == BF16) { CE_FWD(bf16); } else { CE_FWD(f16); }
#undef CE_FWD
  hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(256), 0, st, T, rowloss, loss);
  return hipGetLastError();
}
// Rows on grid.x (no 65535 limit on the number of tokens), column blocks on grid.y.  VEC as for the forward kernel:
// a thread then owns one 16-byte vector of its row.  A row without a valid target has no loss term (ce_fwd gives it
// 0), hence no gradient.
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void ce_bwd_kernel(int V, T* z, int64_t ldz, const int32_t* __restrict__ targets,
                                                     const float* __restrict__ lse, float scale) {
  constexpr int VN = VEC ? Vec<T>::N : 1;
  const int t = blockIdx.x;
  const int c = (blockIdx.y * 256 + threadIdx.x) * VN;
  if (c >= V) return;
  T* p = z + (int64_t)t * ldz + c;
  const int tg = targets[t];
  const bool ok = tg >= 0 && tg < V;
  const float l = lse[t];
  if (VEC) {
    float a[Vec<T>::N], o[Vec<T>::N];
    load_vec(p, a);
#pragma unroll
    for (int i = 0; i < Vec<T>::N; ++i) o[i] = ok ? scale * (expf(a[i] - l) - (c + i == tg ? 1.f : 0.f)) : 0.f;
    store_vec(p, o);
  } else {
    *p = from_f<T>(ok ? scale * (expf(to_f(*p) - l) - (c == tg ? 1.f : 0.f)) : 0.f);
  }
}
hipError_t ce_bwd(hipStream_t st, DType dt, int T, int V, void* z, int64_t ldz, const int32_t* targets,
                  const float* lse, float scale) {
  const int VN = dt == F32 ? 4 : 8;
  const bool vec = V % VN == 0 && ldz % VN == 0 && ((uintptr_t)z & 15) == 0;
  dim3 grid((unsigned)T, (unsigned)cdiv(V, 256 * (vec ? VN : 1))), blk(256);
#define CE_BWD(TT) \
  if (vec) hipLaunchKernelGGL((ce_bwd_kernel<TT, true>), grid, blk, 0, st, V, (TT*)z, ldz, targets, lse, scale); \
  else hipLaunchKernelGGL((ce_bwd_kernel<TT, false>), grid, blk, 0, st, V, (TT*)z, ldz, targets, lse, scale)
  if (dt == F32) { CE_BWD(float); } else if (dt == BF16) { CE_BWD(bf16); } else { CE_BWD(f16); }
#undef CE_BWD
  return hipGetLastError();
}

// ------------------------------------------------------------------ AdamW
__device__ __forceinline__ float adamw_one(float p, float g, float& m, float& v, const AdamW& h) {
  g *= h.grad_scale;
  m = h.beta1 * m + (1.0f - h.beta1) * g;
  v = h.beta2 * v + (1.0f - h.beta2) * g * g;
  const float mhat = m * h.inv_bc1;
  const float vhat = v * h.inv_bc2;
  return p - h.lr * (mhat / (sqrtf(vhat) + h.eps) + h.wd * p);
}

// One float4 of p, g, m, v per lane; reads 16 B/element, writes 12 B (+2 B 16-bit copy; +4 B zeroed grad with h.zero_grad).
// VEC=false is the scalar variant for ranges that are not 16-byte aligned and for the tail.
// W is the element type of the working copy (float: params itself is the master).  With h.skip set and *h.skip
// non-zero (a non-finite gradient was found, loss-scaled fp16 training) nothing but the zeroing of grad happens.
template <typename W, bool VEC>
__global__ __launch_bounds__(256) void adamw_kernel(int64_t n, int64_t begin, void* params, float* master,
                                                    float* grad, float* m, float* v, AdamW h) {
  constexpr bool LOW = sizeof(W) == 2;
  typedef W W4 __attribute__((ext_vector_type(4)));
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * (VEC ? 4 : 1);
  if (i >= n) return;
  const bool skip = h.skip != nullptr && *h.skip != 0;
  float* pm = LOW ? master + i : (float*)params + begin + i;
  if (VEC) {
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    if (skip) {
      if (h.zero_grad) __builtin_nontemporal_store(zero, (f32x4*)(grad + begin + i));
      return;
    }
    // every byte is touched once per step: non-temporal accesses keep the streams out of the caches
    f32x4 p4 = __builtin_nontemporal_load((f32x4*)pm), g4 = __builtin_nontemporal_load((f32x4*)(grad + begin + i)),
          m4 = __builtin_nontemporal_load((f32x4*)(m + i)), v4 = __builtin_nontemporal_load((f32x4*)(v + i));
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      float mm = m4[k], vv = v4[k];
      p4[k] = adamw_one(p4[k], g4[k], mm, vv, h);
      m4[k] = mm;
      v4[k] = vv;
    }
    __builtin_nontemporal_store(p4, (f32x4*)pm);
    __builtin_nontemporal_store(m4, (f32x4*)(m + i));
    __builtin_nontemporal_store(v4, (f32x4*)(v + i));
    if (h.zero_grad) __builtin_nontemporal_store(zero, (f32x4*)(grad + begin + i));
    if (LOW) {
      // The working copy is the rounding of the STORED fp32 value.  Without the barrier the compiler folds the
      // update's last fused multiply-add and the conversion into one mixed-precision instruction that rounds the
      // exact result once, which differs from half(master) whenever the fp32 value lands on a tie.
      W4 b;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        float q = p4[k];
        asm volatile("" : "+v"(q));
        b[k] = (W)q;
      }
      __builtin_nontemporal_store(b, (W4*)((W*)params + begin + i));
    }
  } else {
    if (skip) {
      if (h.zero_grad) grad[begin + i] = 0.f;
      return;
    }
    float mm = m[i], vv = v[i];
    const float pn = adamw_one(*pm, grad[begin + i], mm, vv, h);
    *pm = pn;
    m[i] = mm;
    v[i] = vv;
    if (h.zero_grad) grad[begin + i] = 0.f;
    if (LOW) {
      float q = pn;
      asm volatile("" : "+v"(q));   // as above: round the stored value
      ((W*)params)[begin + i] = (W)q;
    }
  }
}

hipError_t adamw(hipStream_t st, DType dt, int64_t n, int64_t begin, void* params, float* master, float* grad,
                 float* m, float* v, const AdamW& h) {
  if (n <= 0) return hipSuccess;
  const bool aligned = (begin % 4) == 0;   // then grad+begin, params+begin share the alignment of the shard arrays
  const int64_t nv = aligned ? (n / 4) * 4 : 0;
  if (nv > 0) {
    dim3 grid((unsigned)cdiv(nv / 4, 256)), blk(256);
    if (dt == BF16) hipLaunchKernelGGL((adamw_kernel<bf16, true>), grid, blk, 0, st, nv, begin, params, master, grad, m, v, h);
    else if (dt == F16) hipLaunchKernelGGL((adamw_kernel<f16, true>), grid, blk, 0, st, nv, begin, params, master, grad, m, v, h);
    else hipLaunchKernelGGL((adamw_kernel<float, true>), grid, blk, 0, st, nv, begin, params, master, grad, m, v, h);
  }
  if (n > nv) {
    const int64_t r = n - nv;
    dim3 grid((unsigned)cdiv(r, 256)), blk(256);
    if (dt == BF16)
      hipLaunchKernelGGL((adamw_kernel<bf16, false>), grid, blk, 0, st, r, begin + nv, params, master + nv, grad, m + nv, v + nv, h);
    else if (dt == F16)
      hipLaunchKernelGGL((adamw_kernel<f16, false>), grid, blk, 0, st, r, begin + nv, params, master + nv, grad, m + nv, v + nv, h);
    else
      hipLaunchKernelGGL((adamw_kernel<float, false>), grid, blk, 0, st, r, begin + nv, params, (float*)nullptr, grad, m + nv, v + nv, h);
  }
  return hipGetLastError();
}

// Sets *flag to 1 when any of g[0..n) is not finite (never clears it): the overflow test of loss-scaled training.
__global__ __launch_bounds__(256) void nonfinite_kernel(const float* __restrict__ g, int64_t n, int* __restrict__ flag) {
  bool bad = false;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const float x = g[i];
    bad |= !(fabsf(x) <= 3.402823466e38f);   // false for inf and for nan
  }
  if (__any(bad) && (threadIdx.x & 63) == 0) atomicOr(flag, 1);
}
hipError_t nonfinite_check(hipStream_t st, const float* g, int64_t n, int* flag) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = cdiv(n, 256 * 8);
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(nonfinite_kernel, dim3((unsigned)blocks), dim3(256), 0, st, g, n, flag);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float* p, int64_t n) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i + 4 <= n) {
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    *(f32x4*)(p + i) = zero;
  } else {
    for (int64_t k = i; k < n; ++k) p[k] = 0.f;
  }
}
hipError_t fill_zero(hipStream_t st, float* p, int64_t n) {
  if (n <= 0) return hipSuccess;
  // peel so that the vector stores are 16-byte aligned
  int64_t head = ((16 - ((uintptr_t)p & 15)) & 15) / 4;
  if (head > n) head = n;
  if (head) hipLaunchKernelGGL(fill_zero_kernel, dim3(1), dim3(256), 0, st, p, head < 4 ? head : 3);
  p += head;
  n -= head;
  if (n > 0) hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)cdiv(cdiv(n, 4), 256)), dim3(256), 0, st, p, n);
  return hipGetLastError();
}

hipError_t copy_bytes(hipStream_t st, void* dst, const void* src, int64_t bytes) {
  return hipMemcpyAsync(dst, src, (size_t)bytes, hipMemcpyDeviceToDevice, st);
}

}  // namespace zs
