// Plain LDS-tiled GEMM with fp32 FMA accumulation.  It serves the fp32 configuration (which may
// not round below fp32 anywhere) and shapes the MFMA kernel does not take (unaligned leading
// dimensions).  64x64x16 tiles, 256 threads, 4x4 outputs per thread, every access bounds-checked.
#include "kernels.h"

#include <vector>

namespace zs {

template <typename T, int TA, int TB>
__global__ __launch_bounds__(256) void gemm_simple_kernel(Gemm g) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int z = blockIdx.z;
  const T* A = (const T*)g.A + (int64_t)z * g.sA;
  const T* B = (const T*)g.B + (int64_t)z * g.sB;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < g.K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int m, k;
      if (TA == 0) { k = tid & 15; m = (tid >> 4) + 16 * i; }
      else { m = tid & 63; k = (tid >> 6) + 4 * i; }
      const int gm = m0 + m, gk = k0 + k;
      float v = 0.f;
      if (gm < g.M && gk < g.K) v = to_f(TA == 0 ? A[(int64_t)gm * g.lda + gk] : A[(int64_t)gk * g.lda + gm]);
      As[k][m] = v;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int n, k;
      if (TB == 0) { n = tid & 63; k = (tid >> 6) + 4 * i; }
      else { k = tid & 15; n = (tid >> 4) + 16 * i; }
      const int gn = n0 + n, gk = k0 + k;
      float v = 0.f;
      if (gn < g.N && gk < g.K) {
        const int seg = g.kseg ? gk / g.kseg : 0;
        const int kk = g.kseg ? gk - seg * g.kseg : gk;
        const T* Bp = B + (int64_t)seg * g.segB;
        v = to_f(TB == 0 ? Bp[(int64_t)kk * g.ldb + gn] : Bp[(int64_t)gn * g.ldb + kk]);
      }
      Bs[k][n] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }

  const T* bias = g.bias ? (const T*)g.bias + (int64_t)z * g.sBias : nullptr;
  const T* R = g.resid ? (const T*)g.resid + (int64_t)z * g.sC : nullptr;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= g.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= g.N) continue;
      float v = acc[i][j];
      if (bias) v += to_f(bias[gn]);
      if (R) v += to_f(R[(int64_t)gm * g.ldr + gn]);
      if (g.c_f32_accum) {
        float* C = (float*)g.C + (int64_t)z * g.sC;
        C[(int64_t)gm * g.ldc + gn] += v;
      } else {
        T* C = (T*)g.C + (int64_t)z * g.sC;
        C[(int64_t)gm * g.ldc + gn] = from_f<T>(v);
      }
    }
  }
}

template <typename T> static hipError_t launch_simple(hipStream_t st, const Gemm& g) {
  dim3 grid((unsigned)cdiv(g.N, 64), (unsigned)cdiv(g.M, 64), (unsigned)g.batch), blk(256);
  if (!g.transA && !g.transB) hipLaunchKernelGGL((gemm_simple_kernel<T, 0, 0>), grid, blk, 0, st, g);
  else if (!g.transA && g.transB) hipLaunchKernelGGL((gemm_simple_kernel<T, 0, 1>), grid, blk, 0, st, g);
  else if (g.transA && !g.transB) hipLaunchKernelGGL((gemm_simple_kernel<T, 1, 0>), grid, blk, 0, st, g);
  else hipLaunchKernelGGL((gemm_simple_kernel<T, 1, 1>), grid, blk, 0, st, g);
  return hipGetLastError();
}

hipError_t gemm_simple(hipStream_t st, DType dt, const Gemm& g) {
  if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return hipSuccess;
  return dt == F32 ? launch_simple<float>(st, g) : dt == BF16 ? launch_simple<bf16>(st, g) : launch_simple<f16>(st, g);
}

int gemm_select(DType dt, const Gemm& g, int force) {
  if (force == GEMM_SIMPLE) return GEMM_SIMPLE;
  return gemm_mfma_supported(dt, g) ? GEMM_MFMA : GEMM_SIMPLE;
}

namespace {

// Part p of a multi-part K range as a product of its own.
Gemm part_of(const Gemm& g, int p) {
  Gemm a = g;
  a.nx = 0; a.K = p < g.nx ? g.kseg : g.K - g.nx * g.kseg; a.kseg = 0;
  if (p > 0) { a.A = g.Ax[p - 1]; a.B = g.Bx[p - 1]; }
  return a;
}

// One launch: the MFMA kernel when it takes the arguments, else the plain kernel (with the rotation and the
// two-part K range done in extra passes).
hipError_t gemm_one(hipStream_t st, DType dt, const Gemm& g, int force) {
  if (gemm_select(dt, g, force) == GEMM_MFMA) return gemm_mfma(st, dt, g);   // rotation fused into its epilogue
  if (g.glu) {   // gated unit: the plain product(s), then the activation kernel over the dense [gate | up] rows
    Gemm p = g;
    p.glu = 0; p.gu = nullptr;
    if (g.glu == 1) { p.batch = 2; p.C = g.gu; p.ldc = g.gu_ld; p.sC = g.gu_up; }
    const hipError_t e = gemm_one(st, dt, p, force);
    if (e != hipSuccess) return e;
    return g.glu == 1 ? swiglu_fwd(st, dt, g.M, g.N, g.gu, g.C) : swiglu_bwd(st, dt, g.M, g.N, g.gu, g.C, g.gu);
  }
  if (g.nx) {   // multi-part K range: one plain product per part
    for (int p = 0; p <= g.nx; ++p) {
      const hipError_t e = gemm_simple(st, dt, part_of(g, p));
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  hipError_t e = gemm_simple(st, dt, g);
  const int elem = dt == F32 ? 4 : 2;
  for (int z = 0; e == hipSuccess && g.rope && z < g.rope_batches && z < g.batch; ++z)
    e = rope_apply(st, dt, g.M, g.rope_S, g.N, g.rope_d, (char*)g.C + (int64_t)z * g.sC * elem, g.ldc, g.rope, 1.0f);
  return e;
}

// The MFMA kernel addresses each operand with 32-bit byte offsets below 2^30.  A bf16 product whose token-sized
// operand is larger (microbatches of more than about 24 k tokens at a 2 x 11008-wide activation) is cut into
// launches that each stay below the limit, instead of falling to the plain kernel:
//   A stored [M, K] (tokens = rows): ranges of rows of A, C and the residual (a multiple of the tile height and,
//     with a fused rotation, of the sequence length, so that row mod S is unchanged);
//   the accumulating product with A stored [K, M] and B [K, N] (tokens = K): ranges of K, each added into C.
// Returns false when the arguments are not of that kind; the caller then runs them as one launch.
constexpr int64_t OPERAND_LIMIT = 1ll << 30;

bool split_rows(const Gemm& g, std::vector<Gemm>& parts) {
  if (g.transA || g.nx || g.lda <= 0) return false;
  if ((int64_t)g.M * g.lda * 2 < OPERAND_LIMIT) return false;
  int64_t unit = 256;
  if (g.rope) {   // least common multiple of the tile height and the sequence length
    int64_t a = unit, b = g.rope_S;
    while (b) { const int64_t t = a % b; a = b; b = t; }
    unit = unit / a * g.rope_S;
  }
  int64_t rows = (OPERAND_LIMIT - 1 - (int64_t)g.K * 2) / (g.lda * 2) / unit * unit;
  if (rows <= 0) return false;
  for (int64_t r0 = 0; r0 < g.M; r0 += rows) {
    Gemm p = g;
    p.M = (int)(g.M - r0 < rows ? g.M - r0 : rows);
    p.A = (const char*)g.A + r0 * g.lda * 2;
    p.C = (char*)g.C + r0 * g.ldc * (g.c_f32_accum ? 4 : 2);
    if (g.resid) p.resid = (const char*)g.resid + r0 * g.ldr * 2;
    if (g.gu) p.gu = (char*)g.gu + r0 * g.gu_ld * 2;
    parts.push_back(p);
  }
  return true;
}

bool split_k(const Gemm& g, std::vector<Gemm>& parts) {
  if (!g.transA || g.transB || !g.c_f32_accum || g.kseg || g.nx || g.lda <= 0 || g.ldb <= 0) return false;
  const int64_t ld = g.lda > g.ldb ? g.lda : g.ldb;
  if ((int64_t)g.K * ld * 2 < OPERAND_LIMIT) return false;
  const int64_t kc = (OPERAND_LIMIT - 1) / (ld * 2) / 64 * 64;
  if (kc <= 0) return false;
  for (int64_t k0 = 0; k0 < g.K; k0 += kc) {
    Gemm p = g;
    p.K = (int)(g.K - k0 < kc ? g.K - k0 : kc);
    p.A = (const char*)g.A + k0 * g.lda * 2;
    p.B = (const char*)g.B + k0 * g.ldb * 2;
    parts.push_back(p);
  }
  return true;
}

}  // namespace

bool gemm_splits(DType dt, const Gemm& g) {
  if (dt == F32 || gemm_mfma_supported(dt, g)) return false;
  std::vector<Gemm> parts;
  if (!(split_rows(g, parts) || split_k(g, parts))) return false;
  for (const Gemm& p : parts)
    if (!gemm_mfma_supported(dt, p)) return false;
  return true;
}

hipError_t gemm(hipStream_t st, DType dt, const Gemm& g, int force) {
  if (g.glu) {   // the fall-back's activation kernel walks dense rows
    if ((g.glu != 1 && g.glu != 2) || !g.gu || !g.C || g.batch != 1 || g.transA || (g.glu == 1) == (g.transB != 0) ||
        g.c_f32_accum || g.bias || g.resid || g.rope || g.kseg || g.nx || g.ldc != g.N || g.gu_ld != 2ll * g.N || g.gu_up != g.N)
      return hipErrorInvalidValue;
  }
  if (dt != F32 && force != GEMM_SIMPLE && !gemm_mfma_supported(dt, g)) {
    std::vector<Gemm> parts;
    if (g.nx) {   // the parts of a multi-part weight gradient on their own, each cut further if it has to be
      for (int p = 0; p <= g.nx; ++p) {
        const hipError_t e = gemm(st, dt, part_of(g, p), force);
        if (e != hipSuccess) return e;
      }
      return hipSuccess;
    }
    if (split_rows(g, parts) || split_k(g, parts)) {
      for (const Gemm& p : parts) {
        const hipError_t e = gemm_one(st, dt, p, force);
        if (e != hipSuccess) return e;
      }
      return hipSuccess;
    }
  }
  return gemm_one(st, dt, g, force);
}

}  // namespace zs
