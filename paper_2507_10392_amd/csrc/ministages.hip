// Several ministages time-multiplexed on one GPU: K stages of one shape whose parameters and optimizer
// state live in page-locked host memory and visit the device two at a time (the ministage that computes
// and the one being prefetched), each with its own optimizer step right after its backward (the paper's
// Sections 4.1.1, 4.1.2, 5.1 and 5.4).  Built on the public stage API; this file adds residency
// management, the copy stream and the ordering between the two streams.
#include "../../include/ministages.h"

#include <hip/hip_runtime.h>

#include <string>
#include <vector>

namespace {

thread_local std::string g_ms_err;

int64_t up256(int64_t n) { return (n + 255) & ~(int64_t)255; }

// Parameters: the ministage that computes and the one being prefetched.  Optimizer state: the one in use, the one
// whose store is still in flight and the one being loaded, so that a slow store delays nobody.
int param_slots(int K) { return K < 2 ? K : 2; }
int state_slots(int K) { return K < 3 ? K : 3; }

struct Sizes {
  int64_t P = 0, shard = 0, E = 0;
  stage_memory smem{};
  ministages_memory m{};
  int64_t st_master = -1, st_m = 0, st_v = 0;   // offsets inside one device optimizer-state slot
};

int sizes_of(const ministages_config* c, Sizes& z, std::string& err) {
  if (!c) { err = "config is NULL"; return STAGE_ERR_ARG; }
  if (c->n_ministages < 1 || c->n_ministages > 4096) { err = "n_ministages must be in 1..4096"; return STAGE_ERR_ARG; }
  const int rc = stage_query(&c->stage, &z.P, &z.smem, nullptr);
  if (rc != STAGE_OK) { err = stage_last_error(nullptr); return rc; }
  const int K = c->n_ministages;
  const bool bf = c->stage.dtype == STAGE_DTYPE_BF16;
  z.E = bf ? 2 : 4;
  z.shard = c->stage.shard_end - c->stage.shard_begin;
  ministages_memory& m = z.m;
  int64_t o = 0;
  m.off_params = o; o = up256(o + z.P * z.E);
  if (bf) { m.off_master = o; o = up256(o + z.shard * 4); } else m.off_master = -1;
  m.off_m = o; o = up256(o + z.shard * 4);
  m.off_v = o; o = up256(o + z.shard * 4);
  m.off_stash = z.smem.host_stash ? o : -1;              // offload_acts: the ministage's boundary activations
  o = up256(o + z.smem.host_stash);
  m.per_stage_host = o;
  m.host_bytes = o * K;
  m.param_slot = up256(z.P * z.E);
  int64_t s = 0;
  if (bf) { z.st_master = s; s = up256(s + z.shard * 4); }
  z.st_m = s; s = up256(s + z.shard * 4);
  z.st_v = s; s = up256(s + z.shard * 4);
  m.state_slot = s;
  m.grad = up256(z.P * 4);
  m.workspace_each = up256(z.smem.activations);          // what waits for the ministage's backward
  m.scratch = z.smem.workspace - m.workspace_each;       // call-local, shared by all ministages
  m.device_bytes = param_slots(K) * m.param_slot + state_slots(K) * m.state_slot + m.grad + (int64_t)K * m.workspace_each + m.scratch;
  m.resident_bytes = (int64_t)K * (z.smem.params + z.smem.grads + z.smem.optim + z.smem.workspace);
  return STAGE_OK;
}

struct Slot {
  int owner = -1;
  bool fresh = false;        // filled by a load that the stage's stream has not waited for yet
  bool stored = false;       // a store read the slot: whoever writes the slot next (a load, the optimizer) waits for store_done
  bool computed = false;     // compute_done has been recorded
  hipEvent_t copy_done = nullptr;      // load stream: the last load into the slot has finished
  hipEvent_t store_done = nullptr;     // store stream: the last store from the slot has finished
  hipEvent_t compute_done = nullptr;   // stage's stream: the last call that used the slot has finished
};

}  // namespace

struct ministages {
  ministages_config cfg;
  Sizes z;
  int K = 0, np = 0, ns = 0;   // ministages, parameter slots, optimizer-state slots
  hipStream_t st = nullptr;
  // Host-to-device and device-to-host copies run side by side.  (A third stream for the small stores of the
  // updated working parameters was tried: with three copy kernels in flight the compute kernels lost 20 %.)
  hipStream_t load_st = nullptr, store_st = nullptr;
  char* host = nullptr;
  char* pslot[2] = {nullptr, nullptr};
  char* sslot[3] = {nullptr, nullptr, nullptr};
  float* grad = nullptr;
  std::vector<stage_t*> stages;
  Slot ps[2], ss[3];
  int grad_owner = -1;       // ministage whose gradients sit in the shared buffer
  int64_t h2d = 0, d2h = 0;
  std::string err;
};

namespace {

int fail(ministages_t* ms, int code, const std::string& msg) { if (ms) ms->err = msg; else g_ms_err = msg; return code; }

bool ok(ministages_t* ms, hipError_t e, const char* what) {
  if (e == hipSuccess) return true;
  ms->err = std::string(what) + ": " + hipGetErrorString(e);
  return false;
}

hipError_t d2h(ministages_t* ms, void* dst, const void* src, int64_t n) {
  return hipMemcpyAsync(dst, src, n, hipMemcpyDeviceToHost, ms->store_st);
}

char* host_of(ministages_t* ms, int k, int64_t off) { return ms->host + (int64_t)k * ms->z.m.per_stage_host + off; }

// Before a load overwrites a slot, everything the stage's stream did with it must be over, and so must the
// store that copies its old content (or an older version of the incoming data) to the host.
bool load_waits(ministages_t* ms, Slot& s) {
  if (s.computed && !ok(ms, hipStreamWaitEvent(ms->load_st, s.compute_done, 0), "stream wait")) return false;
  if (s.stored && !ok(ms, hipStreamWaitEvent(ms->load_st, s.store_done, 0), "stream wait")) return false;
  return true;
}

bool load_params(ministages_t* ms, int k) {
  Slot& s = ms->ps[k % ms->np];
  if (s.owner == k) return true;
  if (!load_waits(ms, s)) return false;
  const int64_t n = ms->z.P * ms->z.E;
  if (!ok(ms, hipMemcpyAsync(ms->pslot[k % ms->np], host_of(ms, k, ms->z.m.off_params), n, hipMemcpyHostToDevice, ms->load_st),
          "parameter load"))
    return false;
  ms->h2d += n;
  s.owner = k; s.fresh = true;
  return ok(ms, hipEventRecord(s.copy_done, ms->load_st), "event record");
}

bool load_state(ministages_t* ms, int k) {
  Slot& s = ms->ss[k % ms->ns];
  if (s.owner == k || ms->z.shard == 0) return true;
  if (!load_waits(ms, s)) return false;
  const Sizes& z = ms->z;
  char* d = ms->sslot[k % ms->ns];
  const int64_t n = z.shard * 4;
  if (z.st_master >= 0 &&
      !ok(ms, hipMemcpyAsync(d + z.st_master, host_of(ms, k, z.m.off_master), n, hipMemcpyHostToDevice, ms->load_st), "state load"))
    return false;
  if (!ok(ms, hipMemcpyAsync(d + z.st_m, host_of(ms, k, z.m.off_m), n, hipMemcpyHostToDevice, ms->load_st), "state load")) return false;
  if (!ok(ms, hipMemcpyAsync(d + z.st_v, host_of(ms, k, z.m.off_v), n, hipMemcpyHostToDevice, ms->load_st), "state load")) return false;
  ms->h2d += n * (z.st_master >= 0 ? 3 : 2);
  s.owner = k; s.fresh = true;
  return ok(ms, hipEventRecord(s.copy_done, ms->load_st), "event record");
}

// The stage's stream is about to use the slot: wait for a load it has not seen yet and, before writing, for a
// store that may still be reading it.
bool compute_waits_for_copy(ministages_t* ms, Slot& s, bool will_write) {
  if (s.fresh) {
    s.fresh = false;
    if (!ok(ms, hipStreamWaitEvent(ms->st, s.copy_done, 0), "stream wait")) return false;
  }
  if (will_write && s.stored && !ok(ms, hipStreamWaitEvent(ms->st, s.store_done, 0), "stream wait")) return false;
  return true;
}

bool mark_computed(ministages_t* ms, Slot& s) {
  s.computed = true;
  return ok(ms, hipEventRecord(s.compute_done, ms->st), "event record");
}

// After ministage k's optimizer step: what it changed goes back to the host block.
bool store_shard(ministages_t* ms, int k) {
  const Sizes& z = ms->z;
  if (z.shard == 0) return true;
  Slot& p = ms->ps[k % ms->np];
  Slot& s = ms->ss[k % ms->ns];
  // s.compute_done was recorded after the step
  if (!ok(ms, hipStreamWaitEvent(ms->store_st, s.compute_done, 0), "stream wait")) return false;
  const int64_t b = ms->cfg.stage.shard_begin, n4 = z.shard * 4, ne = z.shard * z.E;
  char* d = ms->sslot[k % ms->ns];
  if (!ok(ms, d2h(ms, host_of(ms, k, z.m.off_params) + b * z.E, ms->pslot[k % ms->np] + b * z.E, ne), "parameter store"))
    return false;
  // The parameter slot is free for the next load as soon as its shard has left; the optimizer-state slot (and
  // the host block's state) only when the three larger copies are through.  Whoever writes a slot next (a load,
  // the ministage's next optimizer step) waits for its store_done.
  if (!ok(ms, hipEventRecord(p.store_done, ms->store_st), "event record")) return false;
  if (z.st_master >= 0 &&
      !ok(ms, d2h(ms, host_of(ms, k, z.m.off_master), d + z.st_master, n4), "state store"))
    return false;
  if (!ok(ms, d2h(ms, host_of(ms, k, z.m.off_m), d + z.st_m, n4), "state store")) return false;
  if (!ok(ms, d2h(ms, host_of(ms, k, z.m.off_v), d + z.st_v, n4), "state store")) return false;
  ms->d2h += ne + n4 * (z.st_master >= 0 ? 3 : 2);
  p.stored = s.stored = true;
  return ok(ms, hipEventRecord(s.store_done, ms->store_st), "event record");
}

bool check_k(ministages_t* ms, int k) { return k >= 0 && k < ms->K; }

int pass(ministages_t* ms, int k, int rc) {
  if (rc != STAGE_OK) ms->err = stage_last_error(ms->stages[k]);
  return rc;
}

}  // namespace

extern "C" {

int ministages_query(const ministages_config* cfg, ministages_memory* mem) {
  Sizes z;
  std::string err;
  const int rc = sizes_of(cfg, z, err);
  if (rc != STAGE_OK) return fail(nullptr, rc, err);
  if (mem) *mem = z.m;
  return STAGE_OK;
}

int ministages_init(const ministages_config* cfg, void* hip_stream, void* host_state, int64_t host_bytes, void* device_arena,
                    int64_t device_bytes, ministages_t** out) {
  if (out) *out = nullptr;
  if (!out) return fail(nullptr, STAGE_ERR_ARG, "out is NULL");
  Sizes z;
  std::string err;
  int rc = sizes_of(cfg, z, err);
  if (rc != STAGE_OK) return fail(nullptr, rc, err);
  if (!host_state || host_bytes < z.m.host_bytes)
    return fail(nullptr, STAGE_ERR_ARG, "host_state is NULL or smaller than " + std::to_string(z.m.host_bytes) + " bytes");
  if (!device_arena || ((uintptr_t)device_arena & 255) || device_bytes < z.m.device_bytes)
    return fail(nullptr, STAGE_ERR_WORKSPACE, "device_arena is NULL, not 256-byte aligned or smaller than " +
                                                  std::to_string(z.m.device_bytes) + " bytes");
  hipPointerAttribute_t at;
  if (hipPointerGetAttributes(&at, host_state) != hipSuccess) {
    (void)hipGetLastError();
    return fail(nullptr, STAGE_ERR_ARG, "host_state is not page-locked (allocate it with hipHostMalloc)");
  }
  if (at.type != hipMemoryTypeHost) return fail(nullptr, STAGE_ERR_ARG, "host_state is not page-locked host memory");

  ministages_t* ms = new ministages();
  ms->cfg = *cfg; ms->z = z; ms->K = cfg->n_ministages; ms->np = param_slots(ms->K); ms->ns = state_slots(ms->K);
  ms->st = (hipStream_t)hip_stream;
  ms->host = (char*)host_state;
  char* p = (char*)device_arena;
  for (int i = 0; i < ms->np; ++i) { ms->pslot[i] = p; p += z.m.param_slot; }
  for (int i = 0; i < ms->ns; ++i) { ms->sslot[i] = p; p += z.m.state_slot; }
  ms->grad = (float*)p; p += z.m.grad;
  char* scratch = p; p += z.m.scratch;                    // one call-local scratch buffer for all ministages
  auto bail = [&](int code, const std::string& msg) {
    ministages_destroy(ms);
    return fail(nullptr, code, msg);
  };
  hipError_t e = hipStreamCreateWithFlags(&ms->load_st, hipStreamNonBlocking);   // default priority, both
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&ms->store_st, hipStreamNonBlocking);
  for (Slot* s : {&ms->ps[0], &ms->ps[1], &ms->ss[0], &ms->ss[1], &ms->ss[2]}) {
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->copy_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->store_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->compute_done, hipEventDisableTiming);
  }
  if (e == hipSuccess) e = hipMemsetAsync(ms->grad, 0, z.P * 4, ms->st);
  if (e != hipSuccess) return bail(STAGE_ERR_DEVICE, std::string("ministages_init: ") + hipGetErrorString(e));
  for (int k = 0; k < ms->K; ++k) {
    char* sd = ms->sslot[k % ms->ns];
    stage_t* s = nullptr;
    rc = stage_init_split(&cfg->stage, hip_stream, ms->pslot[k % ms->np],
                          z.st_master >= 0 && z.shard > 0 ? (float*)(sd + z.st_master) : nullptr, ms->grad,
                          z.shard > 0 ? (float*)(sd + z.st_m) : nullptr, z.shard > 0 ? (float*)(sd + z.st_v) : nullptr, p,
                          z.m.workspace_each, scratch, z.m.scratch, &s);
    if (rc != STAGE_OK) return bail(rc, std::string("stage_init of ministage ") + std::to_string(k) + ": " + stage_last_error(nullptr));
    ms->stages.push_back(s);
    if (z.m.off_stash >= 0) {
      rc = stage_attach_host_stash(s, host_of(ms, k, z.m.off_stash), z.smem.host_stash);
      if (rc != STAGE_OK) return bail(rc, std::string("host stash of ministage ") + std::to_string(k) + ": " + stage_last_error(s));
    }
    p += z.m.workspace_each;
  }
  if (!load_params(ms, 0)) { const std::string m2 = ms->err; return bail(STAGE_ERR_DEVICE, m2); }
  *out = ms;
  return STAGE_OK;
}

int ministages_forward(ministages_t* ms, int32_t k, int32_t mb, const void* x_or_ids, void* y_out, const int32_t* targets,
                       float* loss_out) {
  if (!ms) return STAGE_ERR_ARG;
  if (!check_k(ms, k)) return fail(ms, STAGE_ERR_ARG, "ministage index out of range");
  Slot& s = ms->ps[k % ms->np];
  if (!load_params(ms, k) || !compute_waits_for_copy(ms, s, false)) return STAGE_ERR_DEVICE;
  const int rc = stage_forward(ms->stages[k], mb, x_or_ids, y_out, targets, loss_out);
  if (!mark_computed(ms, s)) return STAGE_ERR_DEVICE;
  // the next ministage of the forward order travels while this one computes
  if (rc == STAGE_OK && k + 1 < ms->K && !load_params(ms, k + 1)) return STAGE_ERR_DEVICE;
  return pass(ms, k, rc);
}

int ministages_backward(ministages_t* ms, int32_t k, int32_t mb, const void* dy, void* dx_out, float loss_scale) {
  if (!ms) return STAGE_ERR_ARG;
  if (!check_k(ms, k)) return fail(ms, STAGE_ERR_ARG, "ministage index out of range");
  if (ms->grad_owner >= 0 && ms->grad_owner != k)
    return fail(ms, STAGE_ERR_STATE, "the gradient buffer still holds ministage " + std::to_string(ms->grad_owner) +
                                         "'s gradients: run its optimizer step first");
  Slot& s = ms->ps[k % ms->np];
  if (!load_params(ms, k) || !compute_waits_for_copy(ms, s, false)) return STAGE_ERR_DEVICE;
  const int rc = stage_backward(ms->stages[k], mb, dy, dx_out, loss_scale);
  if (!mark_computed(ms, s)) return STAGE_ERR_DEVICE;
  if (rc == STAGE_OK) {
    ms->grad_owner = k;
    // what the reverse order needs next: this ministage's optimizer state, the previous ministage's parameters
    if (!load_state(ms, k)) return STAGE_ERR_DEVICE;
    if (k > 0 && !load_params(ms, k - 1)) return STAGE_ERR_DEVICE;
  }
  return pass(ms, k, rc);
}

int ministages_accumulate(ministages_t* ms, int32_t k, int32_t mb) {
  if (!ms) return STAGE_ERR_ARG;
  if (!check_k(ms, k)) return fail(ms, STAGE_ERR_ARG, "ministage index out of range");
  return pass(ms, k, stage_accumulate(ms->stages[k], mb));
}

int ministages_optimizer_step(ministages_t* ms, int32_t k, int64_t t, float grad_scale) {
  if (!ms) return STAGE_ERR_ARG;
  if (!check_k(ms, k)) return fail(ms, STAGE_ERR_ARG, "ministage index out of range");
  if (ms->grad_owner >= 0 && ms->grad_owner != k)
    return fail(ms, STAGE_ERR_STATE, "the gradient buffer holds ministage " + std::to_string(ms->grad_owner) + "'s gradients");
  Slot& p = ms->ps[k % ms->np];
  Slot& s = ms->ss[k % ms->ns];
  if (!load_params(ms, k) || !load_state(ms, k)) return STAGE_ERR_DEVICE;
  if (!compute_waits_for_copy(ms, p, true) || !compute_waits_for_copy(ms, s, true)) return STAGE_ERR_DEVICE;
  const int rc = stage_optimizer_step(ms->stages[k], t, grad_scale);
  if (!mark_computed(ms, p) || !mark_computed(ms, s)) return STAGE_ERR_DEVICE;
  if (rc != STAGE_OK) return pass(ms, k, rc);
  ms->grad_owner = -1;
  if (!store_shard(ms, k)) return STAGE_ERR_DEVICE;
  return STAGE_OK;
}

stage_t* ministages_stage(ministages_t* ms, int32_t k) { return ms && check_k(ms, k) ? ms->stages[k] : nullptr; }

int ministages_traffic(const ministages_t* ms, int64_t* h2d_bytes, int64_t* d2h_bytes) {
  if (!ms) return STAGE_ERR_ARG;
  if (h2d_bytes) *h2d_bytes = ms->h2d;
  if (d2h_bytes) *d2h_bytes = ms->d2h;
  return STAGE_OK;
}

const char* ministages_last_error(const ministages_t* ms) { return ms ? ms->err.c_str() : g_ms_err.c_str(); }

void ministages_destroy(ministages_t* ms) {
  if (!ms) return;
  for (hipStream_t c : {ms->load_st, ms->store_st})
    if (c) (void)hipStreamSynchronize(c);   // no copy may outlive the caller's buffers
  for (stage_t* s : ms->stages) stage_destroy(s);
  for (Slot* s : {&ms->ps[0], &ms->ps[1], &ms->ss[0], &ms->ss[1], &ms->ss[2]}) {
    if (s->copy_done) (void)hipEventDestroy(s->copy_done);
    if (s->store_done) (void)hipEventDestroy(s->store_done);
    if (s->compute_done) (void)hipEventDestroy(s->compute_done);
  }
  for (hipStream_t c : {ms->load_st, ms->store_st})
    if (c) (void)hipStreamDestroy(c);
  delete ms;
}

}  // extern "C"
