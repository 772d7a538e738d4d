/*
 * Several ministages time-multiplexed on one GPU (part of libstage, C ABI).
 *
 * The paper assigns several small "ministages" to each GPU and runs them GPipe-style: the forward pass of
 * all microbatches of ministage 0, then of ministage 1, ..., and the backward passes in the reverse order
 * (Section 4.1.1).  Because a ministage's microbatches run together, the ministages that are not running are
 * kept in CPU memory and only two are on the GPU at a time: the one that computes and the next one, which is
 * prefetched meanwhile (Section 4.1.1, Section 5.1).  Each ministage has its own optimizer, which runs on the
 * GPU as soon as that ministage's backward is complete, after which its gradients are freed (Section 4.1.2,
 * Section 5.1, Section 5.4); copies use their own stream so that they do not block compute (Section 5.4).
 *
 * This object reduces that mechanism to what one GPU shows.  It owns K stage_t objects of one shape
 * (include/stage.h) and moves their state between a caller-owned page-locked host block, where all of it
 * lives between uses, and a caller-owned device arena that holds
 *     2 parameter slots            (working parameters of the running and of the prefetched ministage),
 *     3 optimizer-state slots      (fp32 master, m, v of the shard: the one in use, the one whose store is
 *                                   still in flight, the one being loaded),
 *     1 fp32 gradient buffer       (shared: a ministage's gradients are dropped by its optimizer step
 *                                   before the next ministage's backward starts),
 *     K activation workspaces      (each ministage's activations wait for its backward; with offload_acts two
 *                                   microbatch slots each, the rest in the host block),
 *     1 scratch buffer             (call-local, shared by all ministages).
 * Ministage k uses parameter slot k mod 2 and optimizer-state slot k mod 3 (fewer slots when K is smaller).
 *
 * Host block layout: ministage k occupies [k * per_stage_host, (k+1) * per_stage_host); inside it, at the
 * offsets ministages_query reports, the working parameters elem[P], then for the shard the fp32 master
 * (16-bit dtypes only), m and v, then (offload_acts) the stash of its boundary activations.  The caller fills it before the first call (m = v = 0 for a fresh run); after a
 * ministage's optimizer step and a synchronisation of the device it holds the updated shard (working
 * parameters in [shard_begin, shard_end), master, m, v).  Parameters outside the shard are never written.
 *
 * All calls only enqueue work: kernels on the stream given to ministages_init, copies on two extra streams
 * of default priority that the library creates (one for loads, one for stores, so that a slow store never
 * holds up the load the next kernels wait for); the three are ordered with events, nothing synchronises with
 * the host.  Calls must not be captured into a HIP graph.  Return values are the STAGE_* codes.
 */
#ifndef MINISTAGES_H
#define MINISTAGES_H

#include "stage.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ministages ministages_t;

typedef struct {
  stage_config stage;     /* shape of every ministage; shard_begin/end index one ministage's flat parameters;
                             pair_wgrad, recompute and offload_acts are passed through to every ministage (with
                             offload_acts the host block also holds each ministage's boundary activations) */
  int32_t n_ministages;   /* K >= 1 */
  int32_t reserved;
} ministages_config;

typedef struct {
  int64_t per_stage_host;                        /* bytes of one ministage's host block (multiple of 256) */
  int64_t host_bytes;                            /* K * per_stage_host */
  int64_t off_params, off_master, off_m, off_v;  /* offsets inside one ministage's host block; off_master = -1 for dtype 0 */
  int64_t off_stash;                             /* offload_acts: offset of the ministage's boundary activations, else -1 */
  int64_t param_slot, state_slot, grad, workspace_each, scratch;   /* bytes of one slot / buffer on the device */
  int64_t device_bytes;                          /* arena: min(K,2) param slots + min(K,3) state slots + grad + scratch +
                                                    K activation workspaces, in that order */
  int64_t resident_bytes;                        /* what the same K ministages need when all stay on the GPU:
                                                    K * (params + grads + optimizer state + workspace) */
} ministages_memory;

/* Host-only: validates cfg and reports sizes and offsets. */
int ministages_query(const ministages_config* cfg, ministages_memory* mem);

/* Creates the K ministages.
 *   hip_stream    hipStream_t for all kernels (NULL = the null stream)
 *   host_state    HOST pointer, page-locked (hipHostMalloc), mem.host_bytes, filled by the caller; owned by the
 *                 caller, must outlive the object
 *   device_arena  DEVICE pointer, 256-byte aligned, mem.device_bytes; owned by the caller
 * Clears the gradient buffer and starts loading ministage 0's parameters.  On error *out is NULL. */
int ministages_init(const ministages_config* cfg, void* hip_stream, void* host_state, int64_t host_bytes,
                    void* device_arena, int64_t device_bytes, ministages_t** out);

/* stage_forward / stage_backward / stage_accumulate of ministage k (same arguments and errors).  The first use
 * of a ministage whose parameters are not on the device loads them (the kernels wait for the copy); every
 * forward of ministage k also starts the load of ministage k+1's parameters, every backward that of ministage
 * k-1's parameters and of ministage k's optimizer state, unless they are there already.
 * STAGE_ERR_STATE from ministages_backward if another ministage's gradients are still in the shared gradient
 * buffer (its optimizer step has not run). */
int ministages_forward(ministages_t* ms, int32_t k, int32_t mb, const void* x_or_ids, void* y_out,
                       const int32_t* targets, float* loss_out);
int ministages_backward(ministages_t* ms, int32_t k, int32_t mb, const void* dy, void* dx_out, float loss_scale);
int ministages_accumulate(ministages_t* ms, int32_t k, int32_t mb);

/* stage_optimizer_step of ministage k on the GPU, then the updated shard (working parameters of the shard
 * range, master, m, v) is copied back to the host block, and the shared gradient buffer is free (zero) for
 * the next ministage. */
int ministages_optimizer_step(ministages_t* ms, int32_t k, int64_t t, float grad_scale);

/* The underlying stage of ministage k (for stage_profile / stage_profile_read); owned by ms. */
stage_t* ministages_stage(ministages_t* ms, int32_t k);

/* Summed over the object's life: bytes copied host-to-device and device-to-host. */
int ministages_traffic(const ministages_t* ms, int64_t* h2d_bytes, int64_t* d2h_bytes);

/* host string, valid until the next call on ms; ms may be NULL for errors of query/init */
const char* ministages_last_error(const ministages_t* ms);

/* Waits for the copy streams, then frees the K stages and the object (not the caller's buffers). */
void ministages_destroy(ministages_t* ms);

#ifdef __cplusplus
}
#endif
#endif
