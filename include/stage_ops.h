/*
 * Single-kernel entry points of libstage, used to check each kernel of the stage step against
 * the CPU oracle on its own.  Same conventions as stage.h: device pointers, caller-owned
 * buffers, enqueue-only on the given hipStream_t, int status (STAGE_OK / STAGE_ERR_ARG /
 * STAGE_ERR_DEVICE).  dtype: 0 float, 1 bf16, 2 IEEE half.  Argument checks happen on the host before any
 * launch.  The operations are the steps of one decoder layer's forward and backward pass and of
 * the optimizer update that the paper's training iteration consists of (Section 1: forward pass,
 * backward pass, optimizer update); the formulas are stated with each function.
 */
#ifndef STAGE_OPS_H
#define STAGE_OPS_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/* C[M,N] (op)= sum_k A(m,k) B(k,n) (+ bias[n]) (+ R[m,n]).
 * transA 0: A stored [M,K] row-major, lda its row stride; 1: stored [K,M].
 * transB 0: B stored [K,N]; 1: stored [N,K].  c_f32_accum 0: C has `dtype`, overwritten;
 * 1: C is float and the product is added to it.  bias/resid may be NULL.  batch >= 1 with element
 * strides sA, sB, sC (sC also for resid), sBias.  kseg > 0: K is cut in segments of kseg and segment
 * s reads B from B + s*segB.  impl: 0 automatic, 1 the plain fp32-FMA kernel, 2 the 16-bit MFMA
 * kernel with its own choice of workgroup tile, 3 / 4 the MFMA kernel with the 256x256 / 128x128
 * tile (STAGE_ERR_ARG if the shape/alignment is not supported by the MFMA kernel). */
int stage_op_gemm(void* stream, int32_t dtype, int32_t transA, int32_t transB, int32_t M, int32_t N, int32_t K,
                  const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc, int32_t c_f32_accum,
                  const void* bias, const void* resid, int64_t ldr, int32_t batch, int64_t sA, int64_t sB, int64_t sC,
                  int64_t sBias, int32_t kseg, int64_t segB, int32_t impl);

/* stage_op_gemm with the rotary rotation fused into the store (Llama-style Q and K projections): for
 * batch indices z < rope_batches, adjacent column pairs (2i, 2i+1) of every rope_d-wide head of C are
 * rotated by the angle of rope_table[(row mod rope_S), i] = (cos, sin), after bias and residual and
 * before rounding.  rope_table: float[rope_S, rope_d/2, 2] as written by stage_op_rope_table, 16-byte
 * aligned; NULL = plain stage_op_gemm.  Needs c_f32_accum = 0 and N a multiple of rope_d. */
int stage_op_gemm_rope(void* stream, int32_t dtype, int32_t transA, int32_t transB, int32_t M, int32_t N, int32_t K,
                       const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc, int32_t c_f32_accum,
                       const void* bias, const void* resid, int64_t ldr, int32_t batch, int64_t sA, int64_t sB,
                       int64_t sC, int64_t sBias, int32_t kseg, int64_t segB, int32_t impl, const float* rope_table,
                       int32_t rope_S, int32_t rope_d, int32_t rope_batches);

/* Weight gradients of two microbatches in one product: C[M,N] (float) += A1^T B1 + A2^T B2 with A1 stored
 * [K1,M], A2 [K2,M] (row stride lda), B1 [K1,N], B2 [K2,N] (row stride ldb); batch >= 1 with element strides
 * sA, sB (applied to both parts) and sC.  impl as for stage_op_gemm; the MFMA kernel needs K1 to be a multiple
 * of 128 (STAGE_ERR_ARG otherwise when it is forced), impl 0 falls back to one product per part. */
int stage_op_wgrad_pair(void* stream, int32_t dtype, int32_t M, int32_t N, int32_t K1, int32_t K2, const void* A1,
                        const void* A2, int64_t lda, const void* B1, const void* B2, int64_t ldb, float* C, int64_t ldc,
                        int32_t batch, int64_t sA, int64_t sB, int64_t sC, int32_t impl);

/* The same for up to 16 microbatches: C += sum_p A_p^T B_p over nparts parts, A_parts / B_parts being HOST arrays
 * of nparts device pointers; parts 0..nparts-2 have K_each rows, the last one K_last rows.  The MFMA kernel needs
 * K_each to be a multiple of 128 (when there is more than one part). */
int stage_op_wgrad_parts(void* stream, int32_t dtype, int32_t M, int32_t N, int32_t K_each, int32_t K_last, int32_t nparts,
                         const void* const* A_parts, int64_t lda, const void* const* B_parts, int64_t ldb, float* C,
                         int64_t ldc, int32_t batch, int64_t sA, int64_t sB, int64_t sC, int32_t impl);

/* stage_op_wgrad_parts on the MFMA kernel with the K range of the last, partly filled round of 256x256 tiles cut into
 * chunks of whole parts that run side by side (how the stage runs the weight gradients of a group of microbatches,
 * Section 4.1.2's accumulation over microbatches): chunk 0 adds to C, the other chunks write partial tiles into scratch
 * (device memory, 256-byte aligned, caller-owned, free again when the call's work on the stream has finished), and a
 * second kernel adds them to C in the order of the chunks, so a repeat gives the same bits.  The sum differs from
 * stage_op_wgrad_parts' in rounding order only.  stage_op_wgrad_parts_scratch_bytes (host only) returns the bytes this
 * shape needs: 0 when the tiles fill whole rounds or a cut would not pay, and then scratch may be NULL and the call is
 * stage_op_wgrad_parts with impl 2; a negative STAGE_ERR_ARG for invalid sizes.  STAGE_ERR_ARG when the MFMA kernel does
 * not take the arguments, STAGE_ERR_WORKSPACE when scratch is missing, misaligned or too small. */
int64_t stage_op_wgrad_parts_scratch_bytes(int32_t M, int32_t N, int32_t K_each, int32_t K_last, int32_t nparts, int32_t batch);
int stage_op_wgrad_parts_cut(void* stream, int32_t dtype, int32_t M, int32_t N, int32_t K_each, int32_t K_last, int32_t nparts,
                             const void* const* A_parts, int64_t lda, const void* const* B_parts, int64_t ldb, float* C,
                             int64_t ldc, int32_t batch, int64_t sA, int64_t sB, int64_t sC, void* scratch, int64_t scratch_bytes);

/* The gated FFN unit of the Llama-style layer fused into the store of a product (the layer the paper's Llama
 * workloads are built from, Section 6.1); gu is dense [M, 2N] = [gate | up], a dense [M, N].
 * mode 1 (forward): gate = A Wg and up = A Wu are written, rounded, to gu and silu(gate) * up of the ROUNDED values
 *   to a: exactly what the batched product followed by stage_op_swiglu leaves.  A = x [M,K] (row stride lda); Wg and
 *   Wu are stored [K,N] (row stride ldb), Wu lying sB elements behind Wg (B = Wg).
 * mode 2 (backward): da = A B^T with A = dy [M,K] and B = Wd stored [N,K] (row stride ldb; sB ignored); (gate, up)
 *   in gu are replaced by (dgate, dup) = (da * up * silu'(gate), da * silu(gate)).  a is scratch of M*N elements whose
 *   content is unspecified afterwards (the MFMA kernel keeps da in fp32 and never stores it).
 * impl as for stage_op_gemm; implementations other than the MFMA kernel run the plain product(s) and then the
 * activation kernel.  STAGE_ERR_ARG when a forced MFMA kernel does not take the arguments. */
int stage_op_gemm_glu(void* stream, int32_t dtype, int32_t mode, int32_t M, int32_t N, int32_t K, const void* A, int64_t lda,
                      const void* B, int64_t ldb, int64_t sB, void* a, void* gu, int32_t impl);

/* kind 0: LayerNorm n = (x-mean)/sqrt(var+eps)*g + b (biased variance), saves rstd[T], mean[T].
 * kind 1: RMSNorm n = x/sqrt(mean(x^2)+eps)*g, saves rstd[T].  x, n: [T,H]. */
int stage_op_norm_fwd(void* stream, int32_t dtype, int32_t kind, int32_t T, int32_t H, const void* x, const void* g,
                      const void* b, float eps, void* n, float* rstd, float* mean);
/* dx = (dres ? dres : 0) + J^T dn; dg_part/db_part: float[nblk,H] per-row-block partial sums of
 * dn*xhat and dn (db_part NULL for RMSNorm); nblk <= T. */
int stage_op_norm_bwd(void* stream, int32_t dtype, int32_t kind, int32_t T, int32_t H, const void* dn, const void* x,
                      const void* g, const float* rstd, const float* mean, const void* dres, void* dx,
                      float* dg_part, float* db_part, int32_t nblk);

/* In-place rotation of adjacent pairs (2i,2i+1) of every d-wide head in a[T,ncols] (row stride ld)
 * by sign * (t mod S) * base^(-2i/d).  table: float[S, d/2, 2] scratch that receives (cos, sin). */
int stage_op_rope(void* stream, int32_t dtype, int32_t T, int32_t S, int32_t ncols, int32_t d, void* a, int64_t ld,
                  float base, float sign, float* table);

/* table[s, i] = (cos, sin)(s * base^(-2i/d)) for s < S, i < d/2, angles formed in double precision. */
int stage_op_rope_table(void* stream, int32_t S, int32_t d, float base, float* table);

/* GELU(z) = z*Phi(z) (erf form) and its derivative; SwiGLU a = silu(gate)*up with gu = [gate | up] [T,2F]. */
int stage_op_gelu(void* stream, int32_t dtype, int64_t n, const void* z, const void* da, void* out, int32_t backward);
int stage_op_swiglu(void* stream, int32_t dtype, int32_t T, int32_t F, const void* gu, const void* da, void* out,
                    int32_t backward);

/* Causal softmax attention per (sequence, head): o_i = sum_{j<=i} softmax_j(q_i.k_j/sqrt(d)) v_j.
 * q, k, v: first elements of [mb*S, nh*d] blocks with row stride ld; o row stride ldo;
 * lse: float[mb,nh,S] = log sum_j exp(s_ij).  impl: 0 auto, 1 wave-per-row kernel, 2 MFMA kernel. */
int stage_op_attention_fwd(void* stream, int32_t dtype, int32_t mb, int32_t S, int32_t nh, int32_t d, const void* q,
                           const void* k, const void* v, int64_t ld, void* o, int64_t ldo, float* lse, int32_t impl);
/* Gradients dq, dk, dv (row stride ldd) from dout; delta: float[mb,nh,S] scratch. */
int stage_op_attention_bwd(void* stream, int32_t dtype, int32_t mb, int32_t S, int32_t nh, int32_t d, const void* q,
                           const void* k, const void* v, int64_t ld, const void* o, const void* dout, int64_t ldo,
                           const float* lse, float* delta, void* dq, void* dk, void* dv, int64_t ldd, int32_t impl);

/* stage_op_attention_bwd whose dq and dk are rotated back by the rotary angles before they are stored
 * (gradients of the un-rotated projections): pair (2i, 2i+1) of every head by -angle(s, i), with
 * rope_table as for stage_op_gemm_rope (rope_S = S, rope_d = d); NULL = plain stage_op_attention_bwd. */
int stage_op_attention_bwd_rope(void* stream, int32_t dtype, int32_t mb, int32_t S, int32_t nh, int32_t d, const void* q,
                                const void* k, const void* v, int64_t ld, const void* o, const void* dout, int64_t ldo,
                                const float* lse, float* delta, void* dq, void* dk, void* dv, int64_t ldd, int32_t impl,
                                const float* rope_table);

/* stage_op_attention_bwd for callers that cannot allocate device memory (code under HIP graph capture, serving
 * loops, harnesses that forbid hipMalloc) and therefore have no delta buffer to pass: the row sums delta[mb, nh, S]
 * live in a fixed device array inside the library (STAGE_OP_NOALLOC_MAX_ROWS floats = 4 MiB, held by every GPU the
 * library runs on until the process ends).  Same kernels, same results bit for bit as stage_op_attention_bwd; all other
 * arguments as there.  The call allocates and frees nothing.  The GPU that owns `stream` must be the current device.
 * STAGE_ERR_WORKSPACE if mb * nh * S exceeds STAGE_OP_NOALLOC_MAX_ROWS (nothing is enqueued); STAGE_ERR_DEVICE if the
 * array's device address cannot be obtained.  All calls on one GPU share the one array: calls whose work may overlap
 * on that GPU (different streams without ordering between them) race on it; calls on one stream are safe. */
#define STAGE_OP_NOALLOC_MAX_ROWS (1 << 20)
int stage_op_attention_bwd_noalloc(void* stream, int32_t dtype, int32_t mb, int32_t S, int32_t nh, int32_t d, const void* q,
                                   const void* k, const void* v, int64_t ld, const void* o, const void* dout, int64_t ldo,
                                   const float* lse, void* dq, void* dk, void* dv, int64_t ldd, int32_t impl);

/* x[t,:] = E[ids[t],:] ; dE[id,:] += sum of dx rows of the tokens carrying id (token order). */
int stage_op_embed(void* stream, int32_t dtype, int32_t T, int32_t H, int32_t V, const int32_t* ids, const void* E,
                   void* x, const void* dx, float* dE, int32_t backward);
/* forward: lse[t], rowloss[t] = lse[t]-z[t,target], *loss = mean_t rowloss.  backward (in place):
 * z[t,j] = scale*(exp(z[t,j]-lse[t]) - [j==target[t]]). */
int stage_op_cross_entropy(void* stream, int32_t dtype, int32_t T, int32_t V, void* z, int64_t ldz,
                           const int32_t* targets, float* lse, float* rowloss, float* loss, float scale,
                           int32_t backward);

/* Measurement aid, not a step of the path: what the matrix cores sustain when nothing else happens.  One workgroup of
 * 8 waves per CU (256 workgroups) runs `iters` times the inner loop of the GEMM's 128 x 64 wave tile on operands held in
 * registers - per wave and iteration 16 MFMAs of 32x32x16 (shape = 32) or 32 MFMAs of 16x16x32 (shape = 16), i.e.
 * 2 * 128 * 64 * 32 flops - with no LDS or memory access inside the loop.  The MI355X runs such a loop at its power limit,
 * so flops / time is the rate a bf16 GEMM can approach on it; `bench.py --mfma-ceiling` times it (profiles/mfma_sustained_rate.txt).
 * operands: device, 65536 bytes of bf16 values (read once; random values give the operand switching of a real product);
 * sink: device, 256 * 512 floats (one sum per thread, written once, so that the loop is not optimised away).
 * Total flops of a call: iters * 2 * 128 * 64 * 32 * 8 waves * 256 workgroups.  Enqueues one kernel on `stream`;
 * STAGE_ERR_ARG for another shape, iters < 1 or a null pointer. */
int stage_op_mfma_rate(void* stream, int32_t shape, int32_t iters, const void* operands, float* sink);

/* Measurement aid, not a step of the path: what one LDS access pattern costs.  One workgroup of 8 waves; every wave
 * issues `iters` x 8 wave-wide reads in which lane l reads at byte offset lane_offset[l] of the workgroup's 64 KB of LDS
 * (plus shifts that are the same for all lanes): kind 0 = 16 bytes per lane (ds_read_b128), kind 1 = the 8-byte
 * transposing read of gfx950 (ds_read_b64_tr_b16).  cycles[0] receives the workgroup's cycle count for all of it, so
 * cycles[0] / (iters * 8 * 8) is the LDS time per wave read; bank conflicts raise it above the pattern-free 4.6 (kind 0) or
 * 3.6 (kind 1).  The slab layouts of the GEMM were chosen with it (`bench.py --lds-patterns`, profiles/lds_access_patterns.txt).
 * lane_offset_host: host, 64 offsets, each a multiple of 16 (kind 0) or 8 (kind 1) and at most 20 976 (checked here, since
 * the kernel reads at them: STAGE_ERR_ARG otherwise); lane_offset: device, the same 64 values; cycles: device, 2 x int64
 * (the second word is a checksum that keeps the reads alive).  Enqueues one kernel on `stream`. */
int stage_op_lds_probe(void* stream, int32_t kind, const int32_t* lane_offset_host, const int32_t* lane_offset, int32_t iters,
                       int64_t* cycles);

/* AdamW with decoupled weight decay, step t >= 1, on n elements starting at flat index `begin`
 * (formula in stage.h).  dtype 1: master/m/v are float[n], grad float[>=begin+n], params bf16;
 * dtype 0: master NULL, params float.  grad[begin..begin+n) is zeroed. */
int stage_op_adamw(void* stream, int32_t dtype, int64_t n, int64_t begin, void* params, float* master, float* grad,
                   float* m, float* v, float lr, float beta1, float beta2, float eps, float wd, int64_t t,
                   float grad_scale);

#ifdef __cplusplus
}
#endif
#endif
