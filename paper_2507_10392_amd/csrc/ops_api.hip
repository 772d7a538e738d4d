// C-ABI wrappers around single kernels (declared in include/stage_ops.h).
#include "../../include/stage.h"
#include "../../include/stage_ops.h"
#include "kernels.h"

#include <cmath>
#include <mutex>

using namespace zs;

namespace {
int rc(hipError_t e) { return e == hipSuccess ? STAGE_OK : STAGE_ERR_DEVICE; }
bool dt_ok(int d) { return d == 0 || d == 1 || d == 2; }
int vec_of(int d) { return d == 0 ? 4 : 8; }

// Scratch of stage_op_attention_bwd_noalloc: the row sums delta[mb, nh, S] that the dQ kernel leaves for the dK/dV
// kernel.  A file-scope device array, so every GPU the library runs on holds one copy of it (4 MiB) from the moment
// the code object is loaded until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress, not a device address: kernels are given the address that call returns for the CURRENT device,
// looked up once per device and kept.
static __device__ __align__(256) float scratch[STAGE_OP_NOALLOC_MAX_ROWS];
constexpr int MAX_DEVICES = 64;
float* scratch_ptr[MAX_DEVICES] = {};
std::mutex scratch_mu;

// Device address of `scratch` on the current device, or nullptr (no current device, or the lookup failed).
float* scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
  std::lock_guard<std::mutex> lock(scratch_mu);
  if (!scratch_ptr[dev]) {
    float* p = nullptr;
    if (hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
    scratch_ptr[dev] = p;
  }
  return scratch_ptr[dev];
}
}  // namespace

extern "C" {

int stage_op_gemm_rope(void* stream, int32_t dtype, int32_t transA, int32_t transB, int32_t M, int32_t N, int32_t K,
                       const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc, int32_t c_f32_accum,
                       const void* bias, const void* resid, int64_t ldr, int32_t batch, int64_t sA, int64_t sB,
                       int64_t sC, int64_t sBias, int32_t kseg, int64_t segB, int32_t impl, const float* rope_table,
                       int32_t rope_S, int32_t rope_d, int32_t rope_batches) {
  if (!dt_ok(dtype) || M < 0 || N < 0 || K < 0 || batch < 1 || !A || !B || !C || kseg < 0) return STAGE_ERR_ARG;
  if (kseg > 0 && K % kseg) return STAGE_ERR_ARG;
  Gemm g;
  g.M = M; g.N = N; g.K = K; g.transA = transA != 0; g.transB = transB != 0;
  g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc; g.c_f32_accum = c_f32_accum != 0;
  g.bias = bias; g.resid = resid; g.ldr = ldr; g.batch = batch; g.sA = sA; g.sB = sB; g.sC = sC; g.sBias = sBias;
  g.kseg = kseg; g.segB = segB;
  if (rope_table) {
    if (c_f32_accum || rope_S < 1 || rope_d < 8 || rope_d % 8 || N % rope_d || rope_batches < 0) return STAGE_ERR_ARG;
    g.rope = (const float2*)rope_table; g.rope_S = rope_S; g.rope_d = rope_d; g.rope_batches = rope_batches;
  }
  if (impl < 0 || impl > 4) return STAGE_ERR_ARG;
  if (impl >= GEMM_MFMA && !gemm_mfma_supported((DType)dtype, g)) return STAGE_ERR_ARG;
  if (impl > GEMM_MFMA) gemm_mfma_force_tile(impl - GEMM_MFMA);     // 3, 4: fixed workgroup tile
  const hipError_t e = gemm((hipStream_t)stream, (DType)dtype, g, impl > GEMM_MFMA ? GEMM_MFMA : impl);
  gemm_mfma_force_tile(0);
  return rc(e);
}

int stage_op_wgrad_pair(void* stream, int32_t dtype, int32_t M, int32_t N, int32_t K1, int32_t K2, const void* A1,
                        const void* A2, int64_t lda, const void* B1, const void* B2, int64_t ldb, float* C, int64_t ldc,
                        int32_t batch, int64_t sA, int64_t sB, int64_t sC, int32_t impl) {
  if (!dt_ok(dtype) || M < 1 || N < 1 || K1 < 1 || K2 < 1 || batch < 1 || !A1 || !A2 || !B1 || !B2 || !C) return STAGE_ERR_ARG;
  if (impl < 0 || impl > 4) return STAGE_ERR_ARG;
  Gemm g;
  g.M = M; g.N = N; g.K = K1 + K2; g.transA = 1; g.transB = 0; g.A = A1; g.lda = lda; g.B = B1; g.ldb = ldb;
  g.C = C; g.ldc = ldc; g.c_f32_accum = 1; g.batch = batch; g.sA = sA; g.sB = sB; g.sC = sC;
  g.nx = 1; g.Ax[0] = A2; g.Bx[0] = B2; g.kseg = K1;
  if (impl >= GEMM_MFMA && !gemm_mfma_supported((DType)dtype, g)) return STAGE_ERR_ARG;
  if (impl > GEMM_MFMA) gemm_mfma_force_tile(impl - GEMM_MFMA);
  const hipError_t e = gemm((hipStream_t)stream, (DType)dtype, g, impl > GEMM_MFMA ? GEMM_MFMA : impl);
  gemm_mfma_force_tile(0);
  return rc(e);
}

int stage_op_wgrad_parts(void* stream, int32_t dtype, int32_t M, int32_t N, int32_t K_each, int32_t K_last, int32_t nparts,
                         const void* const* A_parts, int64_t lda, const void* const* B_parts, int64_t ldb, float* C, int64_t ldc,
                         int32_t batch, int64_t sA, int64_t sB, int64_t sC, int32_t impl) {
  if (!dt_ok(dtype) || M < 1 || N < 1 || K_each < 1 || K_last < 1 || nparts < 1 || nparts > GEMM_MAX_PARTS || batch < 1 ||
      !A_parts || !B_parts || !C)
    return STAGE_ERR_ARG;
  if (impl < 0 || impl > 4) return STAGE_ERR_ARG;
  for (int p = 0; p < nparts; ++p)
    if (!A_parts[p] || !B_parts[p]) return STAGE_ERR_ARG;
  Gemm g;
  g.M = M; g.N = N; g.K = K_each * (nparts - 1) + K_last; g.transA = 1; g.transB = 0; g.A = A_parts[0]; g.lda = lda;
  g.B = B_parts[0]; g.ldb = ldb; g.C = C; g.ldc = ldc; g.c_f32_accum = 1; g.batch = batch; g.sA = sA; g.sB = sB; g.sC = sC;
  g.nx = nparts - 1;
  if (g.nx) g.kseg = K_each;
  for (int p = 1; p < nparts; ++p) { g.Ax[p - 1] = A_parts[p]; g.Bx[p - 1] = B_parts[p]; }
  if (impl >= GEMM_MFMA && !gemm_mfma_supported((DType)dtype, g)) return STAGE_ERR_ARG;
  if (impl > GEMM_MFMA) gemm_mfma_force_tile(impl - GEMM_MFMA);
  const hipError_t e = gemm((hipStream_t)stream, (DType)dtype, g, impl > GEMM_MFMA ? GEMM_MFMA : impl);
  gemm_mfma_force_tile(0);
  return rc(e);
}

namespace {
Gemm wgrad_parts_gemm(int32_t M, int32_t N, int32_t K_each, int32_t K_last, int32_t nparts, int64_t lda, int64_t ldb, int64_t ldc,
                      int32_t batch, int64_t sA, int64_t sB, int64_t sC) {
  Gemm g;
  g.M = M; g.N = N; g.K = K_each * (nparts - 1) + K_last; g.transA = 1; g.transB = 0; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  g.c_f32_accum = 1; g.batch = batch; g.sA = sA; g.sB = sB; g.sC = sC;
  g.nx = nparts - 1;
  if (g.nx) g.kseg = K_each;
  return g;
}
}  // namespace

int64_t stage_op_wgrad_parts_scratch_bytes(int32_t M, int32_t N, int32_t K_each, int32_t K_last, int32_t nparts, int32_t batch) {
  if (M < 1 || N < 1 || K_each < 1 || K_last < 1 || nparts < 1 || nparts > GEMM_MAX_PARTS || batch < 1) return -STAGE_ERR_ARG;
  return gemm_mfma_ws_bytes(wgrad_parts_gemm(M, N, K_each, K_last, nparts, M, N, N, batch, 0, 0, 0));
}

int stage_op_wgrad_parts_cut(void* stream, int32_t dtype, int32_t M, int32_t N, int32_t K_each, int32_t K_last, int32_t nparts,
                             const void* const* A_parts, int64_t lda, const void* const* B_parts, int64_t ldb, float* C,
                             int64_t ldc, int32_t batch, int64_t sA, int64_t sB, int64_t sC, void* scratch, int64_t scratch_bytes) {
  if (!dt_ok(dtype) || M < 1 || N < 1 || K_each < 1 || K_last < 1 || nparts < 1 || nparts > GEMM_MAX_PARTS || batch < 1 ||
      !A_parts || !B_parts || !C)
    return STAGE_ERR_ARG;
  for (int p = 0; p < nparts; ++p)
    if (!A_parts[p] || !B_parts[p]) return STAGE_ERR_ARG;
  Gemm g = wgrad_parts_gemm(M, N, K_each, K_last, nparts, lda, ldb, ldc, batch, sA, sB, sC);
  g.A = A_parts[0]; g.B = B_parts[0]; g.C = C;
  for (int p = 1; p < nparts; ++p) { g.Ax[p - 1] = A_parts[p]; g.Bx[p - 1] = B_parts[p]; }
  if (!gemm_mfma_supported((DType)dtype, g)) return STAGE_ERR_ARG;
  const int64_t need = gemm_mfma_ws_bytes(g);
  if (need > 0 && (!scratch || ((uintptr_t)scratch & 255) || scratch_bytes < need)) return STAGE_ERR_WORKSPACE;
  g.ws = need > 0 ? scratch : nullptr; g.ws_bytes = need > 0 ? scratch_bytes : 0;
  return rc(gemm((hipStream_t)stream, (DType)dtype, g, GEMM_MFMA));
}

int stage_op_gemm_glu(void* stream, int32_t dtype, int32_t mode, int32_t M, int32_t N, int32_t K, const void* A, int64_t lda,
                      const void* B, int64_t ldb, int64_t sB, void* a, void* gu, int32_t impl) {
  if (!dt_ok(dtype) || (mode != 1 && mode != 2) || M < 1 || N < 1 || K < 1 || !A || !B || !a || !gu) return STAGE_ERR_ARG;
  if (impl < 0 || impl > 4) return STAGE_ERR_ARG;
  Gemm g;
  g.M = M; g.N = N; g.K = K; g.transB = mode == 2; g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.sB = mode == 1 ? sB : 0;
  g.C = a; g.ldc = N; g.glu = mode; g.gu = gu; g.gu_ld = 2ll * N; g.gu_up = N;
  if (impl >= GEMM_MFMA && !gemm_mfma_supported((DType)dtype, g)) return STAGE_ERR_ARG;
  if (impl > GEMM_MFMA) gemm_mfma_force_tile(impl - GEMM_MFMA);
  const hipError_t e = gemm((hipStream_t)stream, (DType)dtype, g, impl > GEMM_MFMA ? GEMM_MFMA : impl);
  gemm_mfma_force_tile(0);
  return rc(e);
}

int stage_op_gemm(void* stream, int32_t dtype, int32_t transA, int32_t transB, int32_t M, int32_t N, int32_t K,
                  const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc, int32_t c_f32_accum,
                  const void* bias, const void* resid, int64_t ldr, int32_t batch, int64_t sA, int64_t sB, int64_t sC,
                  int64_t sBias, int32_t kseg, int64_t segB, int32_t impl) {
  return stage_op_gemm_rope(stream, dtype, transA, transB, M, N, K, A, lda, B, ldb, C, ldc, c_f32_accum, bias, resid, ldr,
                            batch, sA, sB, sC, sBias, kseg, segB, impl, nullptr, 0, 0, 0);
}

int stage_op_norm_fwd(void* stream, int32_t dtype, int32_t kind, int32_t T, int32_t H, const void* x, const void* g,
                      const void* b, float eps, void* n, float* rstd, float* mean) {
  if (!dt_ok(dtype) || (kind != 0 && kind != 1) || T < 0 || H < 1 || H % vec_of(dtype) || !x || !g || !n || !rstd)
    return STAGE_ERR_ARG;
  if (kind == 0 && (!b || !mean)) return STAGE_ERR_ARG;
  if (T == 0) return STAGE_OK;
  return rc(norm_fwd((hipStream_t)stream, (DType)dtype, kind, T, H, x, g, b, eps, n, rstd, mean));
}

int stage_op_norm_bwd(void* stream, int32_t dtype, int32_t kind, int32_t T, int32_t H, const void* dn, const void* x,
                      const void* g, const float* rstd, const float* mean, const void* dres, void* dx,
                      float* dg_part, float* db_part, int32_t nblk) {
  if (!dt_ok(dtype) || (kind != 0 && kind != 1) || T < 1 || H < 1 || H % vec_of(dtype) || !dn || !x || !g || !rstd ||
      !dx || !dg_part || nblk < 1 || nblk > T)
    return STAGE_ERR_ARG;
  if (kind == 0 && (!mean || !db_part)) return STAGE_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  return rc(norm_bwd_partials(st, (DType)dtype, kind, T, H, dn, x, g, rstd, mean, dres, dx, dg_part, db_part, nblk));
}

int stage_op_rope(void* stream, int32_t dtype, int32_t T, int32_t S, int32_t ncols, int32_t d, void* a, int64_t ld,
                  float base, float sign, float* table) {
  if (!dt_ok(dtype) || T < 0 || S < 1 || d < 2 || d % 8 || ncols % d || !a || !table || !(base > 0.f)) return STAGE_ERR_ARG;
  if (T == 0) return STAGE_OK;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = rope_table(st, S, d, base, (float2*)table);
  if (e == hipSuccess) e = rope_apply(st, (DType)dtype, T, S, ncols, d, a, ld, (const float2*)table, sign);
  return rc(e);
}

int stage_op_rope_table(void* stream, int32_t S, int32_t d, float base, float* table) {
  if (S < 1 || d < 2 || d % 2 || !table || !(base > 0.f)) return STAGE_ERR_ARG;
  return rc(rope_table((hipStream_t)stream, S, d, base, (float2*)table));
}

int stage_op_gelu(void* stream, int32_t dtype, int64_t n, const void* z, const void* da, void* out, int32_t backward) {
  if (!dt_ok(dtype) || n < 0 || n % vec_of(dtype) || !z || !out || (backward && !da)) return STAGE_ERR_ARG;
  if (n == 0) return STAGE_OK;
  return rc(backward ? gelu_bwd((hipStream_t)stream, (DType)dtype, n, z, da, out)
                     : gelu_fwd((hipStream_t)stream, (DType)dtype, n, z, out));
}

int stage_op_swiglu(void* stream, int32_t dtype, int32_t T, int32_t F, const void* gu, const void* da, void* out,
                    int32_t backward) {
  if (!dt_ok(dtype) || T < 0 || F < 1 || F % vec_of(dtype) || !gu || !out || (backward && !da)) return STAGE_ERR_ARG;
  if (T == 0) return STAGE_OK;
  return rc(backward ? swiglu_bwd((hipStream_t)stream, (DType)dtype, T, F, gu, da, out)
                     : swiglu_fwd((hipStream_t)stream, (DType)dtype, T, F, gu, out));
}

int stage_op_attention_fwd(void* stream, int32_t dtype, int32_t mb, int32_t S, int32_t nh, int32_t d, const void* q,
                           const void* k, const void* v, int64_t ld, void* o, int64_t ldo, float* lse, int32_t impl) {
  if (!dt_ok(dtype) || mb < 1 || S < 1 || nh < 1 || d < 8 || d % 8 || d > 256 || !q || !k || !v || !o || !lse)
    return STAGE_ERR_ARG;
  if (impl == ATTN_MFMA && attn_select((DType)dtype, S, d, 0) != ATTN_MFMA) return STAGE_ERR_ARG;
  return rc(attn_fwd((hipStream_t)stream, (DType)dtype, mb, S, nh, d, q, k, v, ld, o, ldo, lse, impl));
}

int stage_op_attention_bwd_rope(void* stream, int32_t dtype, int32_t mb, int32_t S, int32_t nh, int32_t d, const void* q,
                                const void* k, const void* v, int64_t ld, const void* o, const void* dout, int64_t ldo,
                                const float* lse, float* delta, void* dq, void* dk, void* dv, int64_t ldd, int32_t impl,
                                const float* rope_table) {
  if (!dt_ok(dtype) || mb < 1 || S < 1 || nh < 1 || d < 8 || d % 8 || d > 256 || !q || !k || !v || !o || !dout || !lse ||
      !delta || !dq || !dk || !dv)
    return STAGE_ERR_ARG;
  if (impl == ATTN_MFMA && attn_select((DType)dtype, S, d, 0) != ATTN_MFMA) return STAGE_ERR_ARG;
  return rc(attn_bwd((hipStream_t)stream, (DType)dtype, mb, S, nh, d, q, k, v, ld, o, dout, ldo, lse, delta, dq, dk, dv,
                     ldd, (const float2*)rope_table, impl));
}

int stage_op_attention_bwd(void* stream, int32_t dtype, int32_t mb, int32_t S, int32_t nh, int32_t d, const void* q,
                           const void* k, const void* v, int64_t ld, const void* o, const void* dout, int64_t ldo,
                           const float* lse, float* delta, void* dq, void* dk, void* dv, int64_t ldd, int32_t impl) {
  return stage_op_attention_bwd_rope(stream, dtype, mb, S, nh, d, q, k, v, ld, o, dout, ldo, lse, delta, dq, dk, dv, ldd,
                                     impl, nullptr);
}

int stage_op_attention_bwd_noalloc(void* stream, int32_t dtype, int32_t mb, int32_t S, int32_t nh, int32_t d, const void* q,
                                   const void* k, const void* v, int64_t ld, const void* o, const void* dout, int64_t ldo,
                                   const float* lse, void* dq, void* dk, void* dv, int64_t ldd, int32_t impl) {
  if (mb < 1 || S < 1 || nh < 1) return STAGE_ERR_ARG;
  if ((int64_t)mb * nh * S > (int64_t)STAGE_OP_NOALLOC_MAX_ROWS) return STAGE_ERR_WORKSPACE;   // delta would not fit
  float* delta = scratch_on_current_device();
  if (!delta) return STAGE_ERR_DEVICE;
  // Every row of delta that the dK/dV kernel reads is written by this call's dQ (or delta) kernel first, in stream
  // order, so nothing of an earlier call's content needs clearing.
  return stage_op_attention_bwd_rope(stream, dtype, mb, S, nh, d, q, k, v, ld, o, dout, ldo, lse, delta, dq, dk, dv, ldd,
                                     impl, nullptr);
}

int stage_op_embed(void* stream, int32_t dtype, int32_t T, int32_t H, int32_t V, const int32_t* ids, const void* E,
                   void* x, const void* dx, float* dE, int32_t backward) {
  if (!dt_ok(dtype) || T < 0 || H < 1 || H % vec_of(dtype) || V < 1 || !ids) return STAGE_ERR_ARG;
  if (backward ? (!dx || !dE) : (!E || !x)) return STAGE_ERR_ARG;
  if (T == 0) return STAGE_OK;
  return rc(backward ? embed_bwd((hipStream_t)stream, (DType)dtype, T, H, V, ids, dx, dE)
                     : embed_fwd((hipStream_t)stream, (DType)dtype, T, H, V, ids, E, x));
}

int stage_op_cross_entropy(void* stream, int32_t dtype, int32_t T, int32_t V, void* z, int64_t ldz,
                           const int32_t* targets, float* lse, float* rowloss, float* loss, float scale,
                           int32_t backward) {
  if (!dt_ok(dtype) || T < 1 || V < 1 || !z || !targets || !lse) return STAGE_ERR_ARG;
  if (!backward && (!rowloss || !loss)) return STAGE_ERR_ARG;
  return rc(backward ? ce_bwd((hipStream_t)stream, (DType)dtype, T, V, z, ldz, targets, lse, scale)
                     : ce_fwd((hipStream_t)stream, (DType)dtype, T, V, z, ldz, targets, lse, rowloss, loss));
}

int stage_op_adamw(void* stream, int32_t dtype, int64_t n, int64_t begin, void* params, float* master, float* grad,
                   float* m, float* v, float lr, float beta1, float beta2, float eps, float wd, int64_t t,
                   float grad_scale) {
  if (!dt_ok(dtype) || n < 0 || begin < 0 || t < 1) return STAGE_ERR_ARG;
  if (n == 0) return STAGE_OK;
  if (!params || !grad || !m || !v) return STAGE_ERR_ARG;
  if ((dtype != 0) != (master != nullptr)) return STAGE_ERR_ARG;
  AdamW h;
  h.lr = lr; h.beta1 = beta1; h.beta2 = beta2; h.eps = eps; h.wd = wd;
  h.inv_bc1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)t)));
  h.inv_bc2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)t)));
  h.grad_scale = grad_scale;
  return rc(adamw((hipStream_t)stream, (DType)dtype, n, begin, params, master, grad, m, v, h));
}

int stage_op_mfma_rate(void* stream, int32_t shape, int32_t iters, const void* operands, float* sink) {
  if ((shape != 16 && shape != 32) || iters < 1 || !operands || !sink) return STAGE_ERR_ARG;
  return rc(mfma_rate((hipStream_t)stream, shape, iters, operands, sink));
}

int stage_op_lds_probe(void* stream, int32_t kind, const int32_t* lane_offset_host, const int32_t* lane_offset, int32_t iters,
                       int64_t* cycles) {
  if ((kind != 0 && kind != 1) || iters < 1 || !lane_offset_host || !lane_offset || !cycles) return STAGE_ERR_ARG;
  for (int l = 0; l < 64; ++l) {   // the host copy is what is checked: the kernel reads LDS at these offsets
    const int o = lane_offset_host[l];
    if (o < 0 || o > lds_probe_max_offset() || o % (kind == 0 ? 16 : 8)) return STAGE_ERR_ARG;
  }
  return rc(lds_probe((hipStream_t)stream, kind, lane_offset, iters, (long long*)cycles));
}

}  // extern "C"
