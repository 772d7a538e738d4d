/*
 * libstage: the per-(mini)stage training step on one MI355X (gfx950), C ABI.
 *
 * A "stage" is one ministage of the paper's interleaved pipeline: a contiguous
 * block of transformer decoder layers that runs the forward pass of all of its
 * microbatches, then their backward passes (Section 4.1.1), accumulating
 * weight gradients in fp32, and then runs its own optimizer update on the
 * rank's data-parallel (ZeRO-2) shard as soon as its backward is complete,
 * after which its gradients are dropped (Section 4.1.2, Section 5.1).  The
 * optimizer runs on the GPU (Section 5.4).  With per-layer activation
 * checkpointing only the layer-boundary activations are kept between forward
 * and backward and the inside of each layer is recomputed (Section 4.1.3).
 * The four terms of the memory model (Section 4.3, "Memory Model") are what
 * stage_query reports.
 *
 * The paper does not define the layer math or name the optimizer; this library
 * implements the standard GPT (pre-LayerNorm, GELU, biases) and Llama
 * (pre-RMSNorm, SwiGLU, RoPE) decoder layers, causal softmax attention, token
 * embedding, LM head with mean cross entropy, and AdamW with decoupled decay.
 *
 * Conventions
 *  - All buffer arguments are DEVICE pointers unless marked "host".  The caller
 *    allocates and owns every device buffer and the stream; the library never
 *    allocates or frees device memory and keeps only raw pointers.  The opaque
 *    stage_t is host memory owned by the library (stage_destroy frees it).
 *  - Every call only enqueues work on the stream given to stage_init and
 *    returns; there is no hidden synchronisation.
 *  - Return value: STAGE_OK or an error code.  Argument, state and budget errors
 *    are detected on the host before anything is enqueued.  A failed kernel
 *    launch returns STAGE_ERR_DEVICE.  stage_last_error gives a message.
 *  - Flat parameter order: [embed E[V,H]] layer_0 .. layer_{L-1} [final_norm.g[H], head Wh[H,V]].
 *    GPT layer:   ln1.g[H] ln1.b[H] Wqkv[H,3H] bqkv[3H] Wo[H,H] bo[H] ln2.g[H] ln2.b[H] W1[H,F] b1[F] W2[F,H] b2[H]
 *    Llama layer: rms1.g[H] Wq[H,H] Wk[H,H] Wv[H,H] Wo[H,H] rms2.g[H] Wg[H,F] Wu[H,F] Wd[F,H]
 *    Matrices are row-major [in, out] and applied as y = x * W.  Wqkv's columns
 *    are [Q | K | V]; head h owns columns h*d .. (h+1)*d-1 of its block.
 *  - Activations are row-major [T, H] with T = microbatch*seq tokens, token
 *    t = b*seq + s.  dtype 0: float everywhere.  dtype 1: bf16 activations and
 *    working parameters, fp32 master weights, gradients and Adam moments.
 *    dtype 2: the same with IEEE half (fp16) in place of bf16, the mixed precision the
 *    paper trains in (Section 6.1); meant to be used with loss scaling, which stays
 *    with the caller: interior stages receive dy already scaled, the head stage's
 *    loss_scale carries the scale, grad_scale of the optimizer step takes it out
 *    again, stage_set_overflow_flag finds the steps to skip and
 *    stage_loss_scale_update is the usual rule for adapting the scale.
 */
#ifndef STAGE_H
#define STAGE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct stage stage_t;

enum {
  STAGE_OK = 0,
  STAGE_ERR_ARG = 1,        /* bad configuration or argument */
  STAGE_ERR_STATE = 2,      /* call not legal in the current schedule state */
  STAGE_ERR_WORKSPACE = 3,  /* workspace missing, misaligned or too small */
  STAGE_ERR_BUDGET = 4,     /* activations exceed act_budget_bytes */
  STAGE_ERR_DEVICE = 5      /* a HIP call failed */
};

enum { STAGE_ARCH_GPT = 0, STAGE_ARCH_LLAMA = 1 };
enum { STAGE_DTYPE_F32 = 0, STAGE_DTYPE_BF16 = 1, STAGE_DTYPE_F16 = 2 };

typedef struct {
  int32_t arch;              /* STAGE_ARCH_* */
  int32_t dtype;             /* STAGE_DTYPE_* */
  int32_t layers, hidden, heads, ffn, seq, microbatch;
  int32_t max_microbatches;  /* M: forwards that may be outstanding before their backwards */
  int32_t vocab;             /* used when has_embed or has_head */
  int32_t has_embed;         /* 1: stage input is int32 token ids, x = E[ids] */
  int32_t has_head;          /* 1: final RMSNorm, LM head and mean cross entropy close the stage */
  int32_t recompute;         /* 0 keep every intermediate; 1 keep layer inputs only and recompute (Section 4.1.3) */
  int32_t pair_wgrad;        /* g >= 2: the weight-gradient products of a group of g microbatches (at most 16, at most
                                max_microbatches; 1 means 2) run as ONE product per weight over the tokens of all of them:
                                every backward but the one that completes a group (or the last outstanding one) only
                                keeps its operands, and grad_acc is read, added to and written once per group instead
                                of once per microbatch.  grad_acc then holds the complete sum once no forwarded
                                microbatch is outstanding, not after every stage_accumulate.  Costs (g-1) * layers * 5
                                activation-sized buffers of scratch, and with a 16-bit dtype up to 256 MiB more for the
                                products whose tiles beyond whole rounds of workgroups are split over the microbatches
                                of the group (partial sums, added in a fixed order: the same bits on every call).
                                Ignored with recompute, with max_microbatches < 2
                                and when seq*microbatch is no multiple of 128. */
  int64_t act_budget_bytes;  /* 0 = unlimited; otherwise stage_query/stage_init fail with STAGE_ERR_BUDGET
                                when the activation term exceeds it */
  int64_t shard_begin, shard_end; /* [begin, end) in flat parameter index space: the optimizer's range */
  float norm_eps, rope_base;
  float lr, beta1, beta2, adam_eps, weight_decay;
  int32_t offload_acts;      /* 1 (needs recompute = 1): the layer-boundary activations of the forwarded microbatches
                                live in pinned host memory (stage_attach_host_stash); the device keeps two microbatch
                                slots, the one in use and the one being prefetched (Section 4.1.3, Section 5.4) */
} stage_config;

/* Bytes per term of the paper's memory model, plus the library's transient scratch.
 * activations: what is held between a microbatch's forward and its backward, for
 * max_microbatches microbatches.  With recompute=1 and an interior stage this is exactly
 * max_microbatches * layers * (microbatch*seq*hidden*sizeof(elem)) (Section 4.1.3).
 * With offload_acts = 1 the device term shrinks to 2 * layers * (...) (current + prefetched microbatch) and
 * host_stash = max_microbatches * layers * (...) bytes move to the host.
 * scratch: buffers live only inside one call.  workspace = activations + scratch, rounded up. */
typedef struct {
  int64_t params, grads, optim, activations, scratch, workspace;
  int64_t host_stash;  /* offload_acts: bytes of pinned host memory for the boundary activations, else 0 */
} stage_memory;

typedef struct {
  char name[32];
  int64_t offset, rows, cols;
} stage_segment;

/* Host-only.  Validates cfg; writes the parameter count, the memory terms and the number of
 * layout segments (any out pointer may be NULL). */
int stage_query(const stage_config* cfg, int64_t* n_params, stage_memory* mem, int32_t* n_segments);

/* Host-only.  Fills out[0..n_segments) with the flat layout; n_segments must be what stage_query returned. */
int stage_layout(const stage_config* cfg, stage_segment* out, int32_t n_segments);

/* Creates a stage bound to caller-owned device buffers.
 *   hip_stream   hipStream_t (NULL = the null stream)
 *   params       working parameters, elem[P] (float or bf16)
 *   master       fp32[shard_end-shard_begin] master copy of the shard; must be NULL for dtype 0,
 *                where params itself is updated
 *   grad_acc     fp32[P]; must be all zero on entry; holds sum over microbatches of the gradients
 *   adam_m/v     fp32[shard_end-shard_begin]
 *   workspace    at least mem.workspace bytes, 256-byte aligned
 * Enqueues small set-up kernels (tables).  On error *out is NULL. */
int stage_init(const stage_config* cfg, void* hip_stream, void* params, float* master, float* grad_acc,
               float* adam_m, float* adam_v, void* workspace, int64_t workspace_bytes, stage_t** out);

/* stage_init with the call-local part of the workspace in a buffer of its own: workspace then needs only
 * mem.activations bytes (rounded up to 256) and scratch mem.workspace minus that.  Stages of ONE configuration
 * that are bound to the same grad_acc and stream and whose calls never interleave inside a microbatch's forward
 * or backward (the ministages of include/ministages.h) may share one scratch buffer; with pair_wgrad a stage's
 * optimizer step must have run before another stage's backward starts.  scratch = NULL is stage_init. */
int stage_init_split(const stage_config* cfg, void* hip_stream, void* params, float* master, float* grad_acc,
                     float* adam_m, float* adam_v, void* workspace, int64_t workspace_bytes, void* scratch,
                     int64_t scratch_bytes, stage_t** out);

/* offload_acts = 1 only (else STAGE_ERR_ARG): hands the library the pinned host buffer that holds the
 * layer-boundary activations between a microbatch's forward and its backward (Section 4.1.3: with offloading
 * only the current and the next, prefetched, microbatch stay on the GPU).  Must be called once, before the
 * first stage_forward.
 *   host_pinned  HOST pointer, page-locked (hipHostMalloc), at least mem.host_stash bytes; owned by the
 *                caller, must outlive the stage
 * The library creates one extra stream of default priority for the copies and orders it against the stage's
 * stream with events (Section 5.4: separate streams, nothing blocks the compute stream unless data is
 * missing).  After each stage_forward the microbatch's boundary activations are copied to the host; a
 * stage_backward whose microbatch is no longer on the device loads it back, and every stage_backward(mb)
 * starts the load of microbatch mb-1 (the next one in the reverse order of Section 4.1.1) before it enqueues
 * its own kernels.  Any call order that is legal without offloading stays legal and gives the same bits.
 * Calls made in this mode must not be captured into a HIP graph.
 * STAGE_ERR_ARG if the buffer is NULL, too small or not page-locked; STAGE_ERR_STATE if called twice. */
int stage_attach_host_stash(stage_t* s, void* host_pinned, int64_t bytes);

/* Forward of microbatch slot mb in [0, max_microbatches).
 *   x_or_ids  elem[T,H] stage input, or int32[T] token ids when has_embed
 *   y_out     elem[T,H] stage output; may be NULL when has_head
 *   targets   int32[T] (has_head only, else NULL); copied into the stage's workspace by this call, so the caller's
 *             buffer is free again once the call's work on the stream is done
 *   loss_out  device float: the microbatch's mean cross entropy (has_head only, else NULL)
 * Indices are never checked on the host (they live in device memory).  A token id outside [0, vocab) reads as an
 * all-zero embedding row and contributes nothing to the embedding's gradient; a target outside [0, vocab) makes its
 * row an ignored one: it adds 0 to the loss sum (the mean still divides by T) and its logits get a zero gradient,
 * so loss and gradient stay consistent with each other.
 * STAGE_ERR_STATE if slot mb already holds a forward that has not been backpropagated, if a
 * backward of this step is still waiting for its stage_accumulate, or if offload_acts = 1 and no host
 * buffer was attached. */
int stage_forward(stage_t* s, int32_t mb, const void* x_or_ids, void* y_out, const int32_t* targets,
                  float* loss_out);

/* Backward of microbatch slot mb (its forward must be outstanding).
 *   dy         elem[T,H] gradient of the stage output (NULL when has_head)
 *   dx_out     elem[T,H] gradient of the stage input (NULL when has_embed)
 *   loss_scale has_head only: the backward seed is loss_scale * d(mean CE)/dz, e.g. 1/M
 * Matrix gradients are added into grad_acc by the weight-gradient GEMM epilogues; vector
 * gradients (biases, norm gains) are left as per-row-block partial sums for stage_accumulate.
 * STAGE_ERR_STATE if another backward still waits for stage_accumulate. */
int stage_backward(stage_t* s, int32_t mb, const void* dy, void* dx_out, float loss_scale);

/* Completes the accumulation of microbatch mb: reduces the vector-gradient partials of the
 * preceding stage_backward(mb) in a fixed order into grad_acc and releases slot mb. */
int stage_accumulate(stage_t* s, int32_t mb);

/* For callers that captured stage_forward / stage_backward / stage_accumulate calls of n_microbatches
 * complete microbatches into a HIP graph on the stage's stream (the calls only enqueue kernels and one
 * device-to-device copy, so they can be captured once the same sequence has run eagerly): after each
 * replay of that graph, this call does the bookkeeping the captured calls did when they were recorded,
 * so that stage_optimizer_step accepts the step.  Host side only, enqueues nothing.
 * STAGE_ERR_STATE if an eagerly started microbatch is still outstanding. */
int stage_graph_replayed(stage_t* stage, int32_t n_microbatches);

/* AdamW step t (1-based) with decoupled weight decay on flat indices [shard_begin, shard_end):
 *   g' = grad_scale*g;  m = b1*m + (1-b1)*g';  v = b2*v + (1-b2)*g'^2;
 *   p = p - lr*( (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps) + wd*p )
 * on the fp32 master (dtype 1, then params[i] = bf16(master), round-to-nearest-even) or on params
 * (dtype 0).  Parameters outside the shard are left as they are (they would arrive from
 * data-parallel peers).  Then grad_acc is set to zero everywhere.  Legal only when at least
 * one microbatch was accumulated and none is outstanding; otherwise STAGE_ERR_STATE. */
int stage_optimizer_step(stage_t* s, int64_t t, float grad_scale);

/* Loss-scaled training (dtype 2).  Once a device flag is set (NULL = off again), every stage_optimizer_step
 * first tests the shard's accumulated gradients and ORs 1 into *device_flag (int32, caller-owned, cleared by the
 * caller) if any of them is inf or nan; the update kernel reads the flag and, when it is non-zero, leaves
 * parameters, master copy and moments untouched (the gradients are still dropped).  The caller reads the flag
 * after the step, and may OR flags of several stages or ranks into one before the step.
 * stage_loss_scale_update is host-only: the usual dynamic rule - a step that overflowed multiplies the scale by
 * backoff (0 < backoff < 1) and restarts the count; growth_interval steps in a row without overflow multiply it
 * by growth (> 1). */
int stage_set_overflow_flag(stage_t* s, int32_t* device_flag);
int stage_loss_scale_update(float* scale, int32_t* good_steps, int32_t found_inf, float backoff, float growth,
                            int32_t growth_interval);

/* Per-kernel-class timing with HIP events on the stage's stream.  stage_profile(s, 1) starts
 * bracketing every launch with events, stage_profile(s, 0) stops.  stage_profile_read
 * synchronises the recorded events and returns, for up to n classes, the class name, number of
 * launches, summed milliseconds, summed algorithmic flops and summed algorithmic bytes, then
 * clears the records.  Returns the number of classes written (negative on error). */
typedef struct {
  char name[32];
  int64_t launches;
  double ms, flops, bytes;
} stage_kernel_stat;
int stage_profile(stage_t* s, int32_t enable);
int stage_profile_read(stage_t* s, stage_kernel_stat* out, int32_t n);

/* Runtime profile for a planner (Section 4.3, "Profiling": layer runtimes are measured at small batch sizes
 * and a linear model predicts the sizes that were not measured; together with the four memory terms of
 * stage_query this is what the paper's planner consumes).
 *
 * stage_time_layers measures this stage at its configured microbatch size: one untimed and then reps timed
 * rounds of stage_forward + stage_backward + stage_accumulate on slot 0, bracketed by HIP events on the stage's
 * stream.  Arguments as for stage_forward / stage_backward (caller-owned device buffers).  Writes the mean
 * milliseconds of one forward and of one backward (+accumulate) of the whole stage; divide by the layer count
 * for a per-layer figure.  Legal only on a stage with nothing outstanding and nothing accumulated
 * (STAGE_ERR_STATE otherwise); SYNCHRONISES the stream; leaves grad_acc all zero and the schedule state as it
 * found it.
 *
 * stage_fit_linear is host-only: ordinary least squares y = intercept + slope * x over n >= 2 points with at
 * least two distinct x (STAGE_ERR_ARG otherwise); r2 is the coefficient of determination (1 when all y are
 * equal). */
typedef struct {
  double intercept, slope, r2;
} stage_linear_fit;
int stage_time_layers(stage_t* s, const void* x_or_ids, void* y_out, const void* dy, void* dx_out, const int32_t* targets,
                      float* loss_out, int32_t reps, double* fwd_ms, double* bwd_ms);
int stage_fit_linear(const double* x, const double* y, int32_t n, stage_linear_fit* out);

/* host string, valid until the next call on s; s may be NULL for errors of stage_query/init */
const char* stage_last_error(const stage_t* s);

void stage_destroy(stage_t* s);

#ifdef __cplusplus
}
#endif
#endif
