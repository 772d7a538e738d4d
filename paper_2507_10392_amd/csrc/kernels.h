// Host-side launchers of the stage kernels.  All pointers are device pointers; every
// launcher only enqueues on the given stream and returns the launch status.
#pragma once
#include "common.h"

namespace zs {

// C[M,N] (op)= sum_k A(m,k) * B(k,n)  (+ bias[n]) (+ R[m,n])
//   transA = 0: A stored row-major [M,K] (lda = row stride);  1: stored [K,M]
//   transB = 0: B stored row-major [K,N] (ldb = row stride);  1: stored [N,K]
//   c_f32_accum = 0: C has the compute dtype and is overwritten
//                 1: C is float and the product is ADDED to it (weight gradients into grad_acc)
//   batch > 1: operand z uses A + z*sA, B + z*sB, C + z*sC, bias + z*sBias, R + z*sC.
//   kseg > 0: the K range is cut in segments of kseg; segment s reads B from B + s*segB
//             (dgrad through several weight matrices stored one after another).
//   nx > 0 (transA = 1, transB = 0, c_f32_accum = 1 only): the K range consists of nx+1 parts with operands of
//             their own, part 0 from A, B and part p from Ax[p-1], Bx[p-1] (same leading dimensions and batch
//             strides); parts 0..nx-1 have kseg rows each, the last one the remaining K - nx*kseg > 0 rows:
//             C += sum_p A_p^T B_p in one K loop (weight gradients of several microbatches).
//   ws != NULL (nx > 0 only): ws_bytes of scratch that the MFMA path may use when the 256x256 tiles of the product do
//             not fill whole rounds of 256 workgroups: the tiles beyond the whole rounds (the last ones of the kernel's
//             tile order, over all batches) then have their K
//             range cut into chunks of whole parts that run side by side, chunk 0 adding to C and the others writing
//             partial tiles into ws, which a second kernel adds to C in the order of the chunks.  The result differs
//             from the uncut product in rounding order only and is the same on every call.
//   rope != NULL (c_f32_accum = 0 only): for batch indices z < rope_batches the adjacent column pairs of
//             every head (rope_d columns wide) of C are rotated, after bias and residual and before the
//             result is rounded, by the angle table[(row % rope_S) * rope_d/2 + pair] (cos, sin).
//   glu != 0 (16-bit or float, transA = 0, batch = 1, c_f32_accum = 0, no bias / residual / rotation / segments):
//             the gated FFN unit fused into the product.  gu is [M, 2N] = [gate | up] with row stride gu_ld and the
//             up half gu_up columns after the gate half; the dispatcher gemm() takes the dense layout only
//             (gu_ld = 2N, gu_up = N, ldc = N).
//             glu = 1 (transB = 0): B and B + sB are the gate and up projections [K,N]; the call writes both
//               products, rounded, to gu and silu(gate) * up of the ROUNDED values to C[M,N]: what the batched
//               product followed by swiglu_fwd leaves.
//             glu = 2 (transB = 1): the product is da[M,N]; the call replaces (gate, up) in gu by (dgate, dup).
//               C is scratch of [M,N] elements whose content is unspecified afterwards (the fused kernel leaves it
//               alone and uses da unrounded).
constexpr int GEMM_MAX_PARTS = 16;   // parts of a multi-part K range
struct Gemm {
  int M = 0, N = 0, K = 0, transA = 0, transB = 0;
  const void* A = nullptr; int64_t lda = 0;
  const void* B = nullptr; int64_t ldb = 0;
  void* C = nullptr; int64_t ldc = 0;
  int c_f32_accum = 0;
  const void* bias = nullptr;
  const void* resid = nullptr; int64_t ldr = 0;
  int batch = 1; int64_t sA = 0, sB = 0, sC = 0, sBias = 0;
  int kseg = 0; int64_t segB = 0;
  int nx = 0; const void* Ax[GEMM_MAX_PARTS - 1] = {}; const void* Bx[GEMM_MAX_PARTS - 1] = {};
  void* ws = nullptr; int64_t ws_bytes = 0;
  // set by gemm_mfma for the launches of a product that is cut, not by callers: the launch covers tiles
  // tile_base .. tile_base + tile_count - 1 of the order gemm_tile_of (over all batches), each in nchunks chunks of chunk_parts parts
  int chunk_parts = 0, nchunks = 1, tile_base = 0, tile_count = 0;
  const float2* rope = nullptr; int rope_S = 0, rope_d = 0, rope_batches = 0;
  int glu = 0; void* gu = nullptr; int64_t gu_ld = 0, gu_up = 0;
};
// Position `pos` of the MFMA kernels' tile order -> tile row and column: the order walks groups of 8 tile rows column by
// column, so that tiles which run at the same time share A rows and B columns.
__host__ __device__ inline void gemm_tile_of(int pos, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int width = 8 * tiles_n, first = (pos / width) * 8;
  const int gsz = tiles_m - first < 8 ? tiles_m - first : 8;
  tm = first + (pos % width) % gsz;
  tn = (pos % width) / gsz;
}
enum GemmImpl { GEMM_AUTO = 0, GEMM_SIMPLE = 1, GEMM_MFMA = 2 };
// Returns which implementation a call with these arguments runs (GEMM_SIMPLE or GEMM_MFMA).
int gemm_select(DType dt, const Gemm& g, int force);
hipError_t gemm(hipStream_t st, DType dt, const Gemm& g, int force);
// True when gemm() runs the call as several MFMA launches because an operand exceeds the kernel's 2^30-byte range.
bool gemm_splits(DType dt, const Gemm& g);
hipError_t gemm_simple(hipStream_t st, DType dt, const Gemm& g);
bool gemm_mfma_supported(DType dt, const Gemm& g);
hipError_t gemm_mfma(hipStream_t st, DType dt, const Gemm& g);
// Scratch bytes (Gemm::ws) with which gemm_mfma would cut the K range of this product's last round of tiles; 0 when
// it would not (the answer depends on the shape only, not on the pointers).
int64_t gemm_mfma_ws_bytes(const Gemm& g);
// Workgroup tile the MFMA kernel would use: 1 = 256x256 (8 waves), 2 = 128x128 (4 waves); force_tile(0) = automatic.
int gemm_mfma_pick_tile(const Gemm& g);
void gemm_mfma_force_tile(int id);

// kind 0 LayerNorm (mean and rstd saved), 1 RMSNorm (rstd saved).  b and mean may be NULL for RMSNorm.
hipError_t norm_fwd(hipStream_t st, DType dt, int kind, int T, int H, const void* x, const void* g, const void* b,
                    float eps, void* n, float* rstd, float* mean);
// dx = (dres ? dres : 0) + norm'(x)^T dn.  dres may alias dx.
hipError_t norm_bwd(hipStream_t st, DType dt, int kind, int T, int H, const void* dn, const void* x, const void* g,
                    const float* rstd, const float* mean, const void* dres, void* dx);
// norm_bwd plus the partial column sums of the gain (and, for LayerNorm, bias) gradient over row blocks of
// cdiv(T, nblk) rows: part_g[blk, c] = sum_t dn * xhat, part_b[blk, c] = sum_t dn (part_b may be NULL for
// RMSNorm).  For the row lengths of the register-resident kernels this is ONE kernel that reads dn and x once (a
// workgroup per row block); otherwise colsum_partial and norm_bwd one after the other.  Same sums either way.
hipError_t norm_bwd_partials(hipStream_t st, DType dt, int kind, int T, int H, const void* dn, const void* x,
                             const void* g, const float* rstd, const float* mean, const void* dres, void* dx,
                             float* part_g, float* part_b, int nblk);
// part[blk, n] = sum over the rows t of block blk of a[t,n] * (x ? (x[t,n]-mean[t])*rstd[t] : 1)
// (mean may be NULL = 0).  Rows are cut in nblk equal blocks.  part is float[nblk, N].
hipError_t colsum_partial(hipStream_t st, DType dt, int T, int N, const void* a, int64_t lda, const void* x,
                          int64_t ldx, const float* rstd, const float* mean, float* part, int nblk);
struct ReduceJob { const float* part; float* dst; int nblk; int width; };
// dst[c] += sum_blk part[blk, c] for every job, blocks added in increasing order.
hipError_t reduce_partials(hipStream_t st, const ReduceJob* jobs_dev, int njobs, int max_width);

// table[s, i] = (cos, sin)(s * base^(-2i/d)), computed in double precision.
hipError_t rope_table(hipStream_t st, int S, int d, float base, float2* table);
// Rotates adjacent pairs of every head in a[T, ncols] (ld = row stride, heads are d wide) in place;
// token t has position t % S; sign = -1 applies the inverse rotation.
hipError_t rope_apply(hipStream_t st, DType dt, int T, int S, int ncols, int d, void* a, int64_t ld,
                      const float2* table, float sign);

hipError_t gelu_fwd(hipStream_t st, DType dt, int64_t n, const void* z, void* a);
hipError_t gelu_bwd(hipStream_t st, DType dt, int64_t n, const void* z, const void* da, void* dz);
// gu is [T, 2F] = [gate | up]; a is [T, F].  dgu may alias gu.
hipError_t swiglu_fwd(hipStream_t st, DType dt, int T, int F, const void* gu, void* a);
hipError_t swiglu_bwd(hipStream_t st, DType dt, int T, int F, const void* gu, const void* da, void* dgu);

// Causal softmax attention.  q, k, v point at the first element of their [T, nh*d] blocks inside a
// buffer with row stride ld (elements); token t = b*S + s.  lse is float[mb, nh, S].
enum AttnImpl { ATTN_AUTO = 0, ATTN_SIMPLE = 1, ATTN_MFMA = 2 };
int attn_select(DType dt, int S, int d, int force);
hipError_t attn_fwd(hipStream_t st, DType dt, int mb, int S, int nh, int d, const void* q, const void* k,
                    const void* v, int64_t ld, void* o, int64_t ldo, float* lse, int force);
// delta is float[mb, nh, S] scratch.  dq, dk, dv are laid out like q, k, v with row stride ldd.
// rope != NULL: dq and dk are rotated back (angle -table[s, pair]) before they are stored, i.e. they are
// the gradients of the un-rotated projections.
hipError_t attn_bwd(hipStream_t st, DType dt, int mb, int S, int nh, int d, const void* q, const void* k,
                    const void* v, int64_t ld, const void* o, const void* dout, int64_t ldo, const float* lse,
                    float* delta, void* dq, void* dk, void* dv, int64_t ldd, const float2* rope, int force);

// x[t,:] = E[ids[t],:] (rows of ids outside [0,V) give zeros).
hipError_t embed_fwd(hipStream_t st, DType dt, int T, int H, int V, const int32_t* ids, const void* E, void* x);
// dE[id,:] += sum over the tokens with that id, added in increasing token order.
hipError_t embed_bwd(hipStream_t st, DType dt, int T, int H, int V, const int32_t* ids, const void* dx, float* dE);
// lse[t] = logsumexp(z[t,:]); rowloss[t] = lse[t] - z[t,target[t]]; then *loss = mean_t rowloss[t].
hipError_t ce_fwd(hipStream_t st, DType dt, int T, int V, const void* z, int64_t ldz, const int32_t* targets,
                  float* lse, float* rowloss, float* loss);
// z[t,j] <- scale * (exp(z[t,j]-lse[t]) - [j == target[t]])   (scale = loss_scale / T)
hipError_t ce_bwd(hipStream_t st, DType dt, int T, int V, void* z, int64_t ldz, const int32_t* targets,
                  const float* lse, float scale);

struct AdamW { float lr, beta1, beta2, eps, wd, inv_bc1, inv_bc2, grad_scale; const int* skip = nullptr; bool zero_grad = true; };
// Elements i in [0,n): flat parameter index begin+i.  dtype BF16: master/m/v indexed by i, grad and
// params_bf16 by begin+i.  dtype F32: params (float) indexed by begin+i is the master.  grad[begin, begin+n) is
// zeroed when h.zero_grad is set; a caller that clears the whole accumulator anyway leaves that to its fill, which
// as a pure write stream runs at a higher rate than a fifth write stream inside this kernel.
// Register-resident MFMA loop (mfma_rate.hip): `shape` 16 = 16x16x32, 32 = 32x32x16; one 512-thread workgroup per CU, every wave
// issues iters * 32 columns of k on a 128 x 64 tile.  operands: 64 KB of bf16 values, sink: MFMA_RATE_BLOCKS * 512 floats.
constexpr int MFMA_RATE_BLOCKS = 256;
hipError_t mfma_rate(hipStream_t st, int shape, int iters, const void* operands, float* sink);
// LDS access-pattern timer (lds_probe.hip): kind 0 = 16-byte reads, 1 = 8-byte transposing reads; lane_offset: 64 byte offsets
// on the device, each at most lds_probe_max_offset(); cycles[0] = the workgroup's cycles for iters * 8 reads per wave, 8 waves.
int lds_probe_max_offset();
hipError_t lds_probe(hipStream_t st, int kind, const int* lane_offset, int iters, long long* cycles);

hipError_t adamw(hipStream_t st, DType dt, int64_t n, int64_t begin, void* params, float* master, float* grad,
                 float* m, float* v, const AdamW& h);
hipError_t fill_zero(hipStream_t st, float* p, int64_t n);
// *flag |= 1 when any of g[0..n) is inf or nan.
hipError_t nonfinite_check(hipStream_t st, const float* g, int64_t n, int* flag);
hipError_t copy_bytes(hipStream_t st, void* dst, const void* src, int64_t bytes);

}  // namespace zs
