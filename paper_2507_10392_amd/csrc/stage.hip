// Host side of libstage: configuration checks, flat layout, workspace plan, the schedule's
// state machine and the sequencing of kernels for forward, backward, accumulate and the
// optimizer step of one pipeline (mini)stage.  Schedule and memory accounting follow the
// paper's Sections 4.1.1-4.1.3 and its memory model; the layer math is the standard GPT /
// Llama decoder layer.
#include "../../include/stage.h"
#include "kernels.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

using namespace zs;

namespace {

thread_local std::string g_err;  // errors raised before a stage exists

struct Seg { std::string name; int64_t off, rows, cols; };

struct Shape {
  int arch, L, H, nh, d, F, S, mb, T, M, V, dtype;
  bool bf /* 16-bit elements (bf16 or fp16) with an fp32 master copy */, embed, head, recompute, pair, offload;
  int group;   // pair: microbatches whose weight-gradient products share one K loop (2..GEMM_MAX_PARTS)
  int64_t E;  // bytes per element
};

Shape shape_of(const stage_config& c) {
  Shape s;
  s.arch = c.arch; s.L = c.layers; s.H = c.hidden; s.nh = c.heads; s.d = c.heads ? c.hidden / c.heads : 0;
  s.F = c.ffn; s.S = c.seq; s.mb = c.microbatch; s.T = c.seq * c.microbatch; s.M = c.max_microbatches;
  s.V = c.vocab; s.dtype = c.dtype; s.bf = c.dtype != STAGE_DTYPE_F32; s.embed = c.has_embed != 0; s.head = c.has_head != 0;
  s.recompute = c.recompute != 0; s.E = s.bf ? 2 : 4;
  s.offload = c.offload_acts != 0;
  // weight gradients of two microbatches in one product: needs the first one's activations to stay (no
  // recompute), a second microbatch to pair with, and the part boundary on a K slab of the MFMA kernel
  s.pair = c.pair_wgrad != 0 && !s.recompute && s.M >= 2 && s.T % 128 == 0;
  s.group = c.pair_wgrad < 2 ? 2 : c.pair_wgrad;
  if (s.group > GEMM_MAX_PARTS) s.group = GEMM_MAX_PARTS;
  if (s.group > s.M) s.group = s.M;
  return s;
}

std::vector<Seg> make_layout(const stage_config& c) {
  const int64_t H = c.hidden, F = c.ffn, V = c.vocab;
  std::vector<Seg> v;
  int64_t off = 0;
  auto add = [&](const std::string& n, int64_t r, int64_t cc) { v.push_back({n, off, r, cc}); off += r * cc; };
  if (c.has_embed) add("embed.E", V, H);
  for (int l = 0; l < c.layers; ++l) {
    const std::string p = "L" + std::to_string(l) + ".";
    if (c.arch == STAGE_ARCH_GPT) {
      add(p + "ln1.g", 1, H); add(p + "ln1.b", 1, H); add(p + "Wqkv", H, 3 * H); add(p + "bqkv", 1, 3 * H);
      add(p + "Wo", H, H); add(p + "bo", 1, H); add(p + "ln2.g", 1, H); add(p + "ln2.b", 1, H);
      add(p + "W1", H, F); add(p + "b1", 1, F); add(p + "W2", F, H); add(p + "b2", 1, H);
    } else {
      add(p + "rms1.g", 1, H); add(p + "Wq", H, H); add(p + "Wk", H, H); add(p + "Wv", H, H); add(p + "Wo", H, H);
      add(p + "rms2.g", 1, H); add(p + "Wg", H, F); add(p + "Wu", H, F); add(p + "Wd", F, H);
    }
  }
  if (c.has_head) { add("final_norm.g", 1, H); add("head.Wh", H, V); }
  return v;
}

int64_t count_params(const stage_config& c) {
  const int64_t H = c.hidden, F = c.ffn, V = c.vocab;
  int64_t per = c.arch == STAGE_ARCH_GPT ? 4 * H * H + 2 * H * F + 9 * H + F : 4 * H * H + 3 * H * F + 2 * H;
  int64_t n = per * c.layers;
  if (c.has_embed) n += V * H;
  if (c.has_head) n += H + H * V;
  return n;
}

int validate(const stage_config* c, std::string& err) {
  if (!c) { err = "config is NULL"; return STAGE_ERR_ARG; }
  auto bad = [&](const char* m) { err = m; return STAGE_ERR_ARG; };
  if (c->arch != STAGE_ARCH_GPT && c->arch != STAGE_ARCH_LLAMA) return bad("arch must be 0 (GPT) or 1 (Llama)");
  if (c->dtype != STAGE_DTYPE_F32 && c->dtype != STAGE_DTYPE_BF16 && c->dtype != STAGE_DTYPE_F16)
    return bad("dtype must be 0 (fp32), 1 (bf16) or 2 (fp16)");
  if (c->layers < 1 || c->hidden < 8 || c->heads < 1 || c->ffn < 8 || c->seq < 1 || c->microbatch < 1)
    return bad("layers, heads, seq, microbatch must be >= 1 and hidden, ffn >= 8");
  if (c->max_microbatches < 1) return bad("max_microbatches must be >= 1");
  if (c->hidden % c->heads) return bad("hidden must be a multiple of heads");
  const int d = c->hidden / c->heads;
  if (d % 8 || d > 256) return bad("head dim must be a multiple of 8 and at most 256");
  if (c->hidden % 8 || c->ffn % 8) return bad("hidden and ffn must be multiples of 8 (16-byte rows)");
  if ((int64_t)c->seq * c->microbatch > (1 << 24)) return bad("microbatch*seq too large");
  if (c->has_embed || c->has_head) {
    if (c->vocab < 8 || c->vocab % 8) return bad("vocab must be a positive multiple of 8 when has_embed or has_head");
  }
  if (c->recompute != 0 && c->recompute != 1) return bad("recompute must be 0 or 1");
  if (c->offload_acts != 0 && c->offload_acts != 1) return bad("offload_acts must be 0 or 1");
  if (c->offload_acts && !c->recompute) return bad("offload_acts needs recompute = 1 (only layer-boundary activations are offloaded)");
  if (c->pair_wgrad < 0) return bad("pair_wgrad must be >= 0");
  if (c->act_budget_bytes < 0) return bad("act_budget_bytes must be >= 0");
  const int64_t P = count_params(*c);
  if (c->shard_begin < 0 || c->shard_end < c->shard_begin || c->shard_end > P) return bad("shard range outside [0, n_params]");
  if (!(c->norm_eps > 0.f)) return bad("norm_eps must be > 0");
  if (c->arch == STAGE_ARCH_LLAMA && !(c->rope_base > 0.f)) return bad("rope_base must be > 0");
  if (!(c->beta1 >= 0.f && c->beta1 < 1.f && c->beta2 >= 0.f && c->beta2 < 1.f)) return bad("betas must be in [0,1)");
  if (!(c->adam_eps > 0.f) || c->lr < 0.f || c->weight_decay < 0.f) return bad("adam_eps > 0, lr >= 0, weight_decay >= 0 required");
  return STAGE_OK;
}

// ---- workspace plan -------------------------------------------------------------------------
struct LayerActs {  // what a layer's backward needs from its forward
  char *x_in, *n1, *qkv, *o, *x2, *n2, *ff /*[T,2F] gate|up, or [T,F] z*/, *a;
  float *rstd1, *mean1, *rstd2, *mean2, *lse;
};
struct HeadActs { char *y, *nf, *logits; float *rstd, *lse, *rowloss; };

struct Bump {
  char* base; int64_t off = 0;
  explicit Bump(char* b) : base(b) {}
  template <typename P = char> P* take(int64_t bytes) {
    off = (off + 255) & ~(int64_t)255;
    char* p = base ? base + off : nullptr;
    off += bytes;
    return reinterpret_cast<P*>(p);
  }
};



constexpr int MAX_NBLK = 256;   // row blocks of the vector-gradient partial sums: one workgroup each in the fused norm backward, 256 CUs
struct Plan {
  std::vector<LayerActs> acts;      // recompute ? 1 : M*L   (index mb*L + l)
  std::vector<char*> stash;         // recompute: M*L layer inputs; offload: 2*L (index device_slot*L + l)
  std::vector<HeadActs> hacts;      // head: recompute ? 1 : M
  std::vector<char*> hstash;        // head && recompute: M inputs of the final norm; offload: 2
  int dev_slots = 0;                // offload: microbatches resident on the device at a time
  int64_t slot_bytes = 0, host_stash_bytes = 0;   // offload: one microbatch's boundary activations; all of them
  std::vector<int32_t*> ids, targets;  // per slot copies
  // scratch
  char *gA, *gB, *gN, *gO, *gQKV, *gF1, *ytmp;
  std::vector<char*> kdy, kdx2, kdqkv;   // pair_wgrad: per deferred microbatch and layer (index set*L + l), its dy, dx2 and dqkv
  char* kcut = nullptr; int64_t kcut_bytes = 0;   // pair_wgrad: partial tiles of the weight-gradient products whose last round is cut along K
  float* delta; float* lossdump;
  float2* rope;
  float* partials; int64_t partial_floats;
  ReduceJob* jobs; int njobs_cap;
  int nblk;
  int64_t act_bytes = 0, scratch_bytes = 0, total = 0;
};

void plan_layer_acts(Bump& b, const Shape& s, LayerActs& a, bool with_x_in) {
  const int64_t TH = (int64_t)s.T * s.H * s.E;
  a.x_in = with_x_in ? b.take(TH) : nullptr;
  a.n1 = b.take(TH);
  a.qkv = b.take(3 * TH);
  a.o = b.take(TH);
  a.x2 = b.take(TH);
  a.n2 = b.take(TH);
  a.ff = b.take((int64_t)s.T * s.F * s.E * (s.arch == STAGE_ARCH_LLAMA ? 2 : 1));
  a.a = b.take((int64_t)s.T * s.F * s.E);
  a.rstd1 = b.take<float>(4ll * s.T);
  a.rstd2 = b.take<float>(4ll * s.T);
  a.mean1 = s.arch == STAGE_ARCH_GPT ? b.take<float>(4ll * s.T) : nullptr;
  a.mean2 = s.arch == STAGE_ARCH_GPT ? b.take<float>(4ll * s.T) : nullptr;
  a.lse = b.take<float>(4ll * s.mb * s.nh * s.S);
}
void plan_head_acts(Bump& b, const Shape& s, HeadActs& h, bool with_y) {
  const int64_t TH = (int64_t)s.T * s.H * s.E;
  h.y = with_y ? b.take(TH) : nullptr;
  h.nf = b.take(TH);
  h.logits = b.take((int64_t)s.T * s.V * s.E);
  h.rstd = b.take<float>(4ll * s.T);
  h.lse = b.take<float>(4ll * s.T);
  h.rowloss = b.take<float>(4ll * s.T);
}

int64_t vector_widths_per_layer(const Shape& s) {   // summed widths of a layer's vector parameters
  return s.arch == STAGE_ARCH_GPT ? 9ll * s.H + s.F : 2ll * s.H;
}

// One routine both sizes (base == NULL) and assigns the workspace, so the two can never disagree.
// scratch_base != NULL: the call-local part is carved from a buffer of its own (stages of one shape that never
// run at the same time may share it); its layout is the one it has behind the activations.
void make_plan(const stage_config& c, char* base, Plan& p, char* scratch_base = nullptr) {
  const Shape s = shape_of(c);
  const int64_t TH = (int64_t)s.T * s.H * s.E;
  Bump b(base);
  // ---- activations held between forward and backward
  if (s.offload) {
    // Section 4.1.3 with offloading: the microbatch in use and the one being prefetched stay on the device.  One
    // microbatch's tensors (L layer inputs, then the final norm's input of a head stage) are contiguous, so a
    // microbatch moves in one copy.
    p.dev_slots = s.M < 2 ? s.M : 2;
    p.slot_bytes = (s.L + (s.head ? 1 : 0)) * TH;
    p.host_stash_bytes = (int64_t)s.M * p.slot_bytes;
    p.stash.resize((size_t)p.dev_slots * s.L);
    if (s.head) p.hstash.resize(p.dev_slots);
    char* blockp = b.take((int64_t)p.dev_slots * p.slot_bytes);
    for (int k = 0; k < p.dev_slots; ++k) {
      char* q = blockp ? blockp + (int64_t)k * p.slot_bytes : nullptr;
      for (int l = 0; l < s.L; ++l) p.stash[(size_t)k * s.L + l] = q ? q + (int64_t)l * TH : nullptr;
      if (s.head) p.hstash[k] = q ? q + (int64_t)s.L * TH : nullptr;
    }
  } else if (s.recompute) {
    p.stash.resize((size_t)s.M * s.L);
    // exactly M*L tensors of T*H elements, packed (Section 4.1.3's formula); TH is a multiple of 16 bytes
    char* blockp = b.take((int64_t)s.M * s.L * TH);
    for (int i = 0; i < s.M * s.L; ++i) p.stash[i] = blockp ? blockp + (int64_t)i * TH : nullptr;
    if (s.head) {
      p.hstash.resize(s.M);
      for (int i = 0; i < s.M; ++i) p.hstash[i] = b.take(TH);
    }
  } else {
    p.acts.resize((size_t)s.M * s.L);
    for (auto& a : p.acts) plan_layer_acts(b, s, a, true);
    if (s.head) { p.hacts.resize(s.M); for (auto& h : p.hacts) plan_head_acts(b, s, h, true); }
  }
  if (s.embed) { p.ids.resize(s.M); for (auto& q : p.ids) q = b.take<int32_t>(4ll * s.T); }
  if (s.head) { p.targets.resize(s.M); for (auto& q : p.targets) q = b.take<int32_t>(4ll * s.T); }
  p.act_bytes = b.off;
  const int64_t act_end = (b.off + 255) & ~(int64_t)255;
  if (scratch_base) b = Bump(scratch_base);
  // ---- scratch live inside one call
  if (s.recompute) {
    p.acts.resize(1);
    plan_layer_acts(b, s, p.acts[0], false);
    if (s.head) { p.hacts.resize(1); plan_head_acts(b, s, p.hacts[0], false); }
  }
  p.gA = b.take(TH); p.gB = b.take(TH); p.gN = b.take(TH); p.gO = b.take(TH);
  p.gQKV = b.take(3 * TH);
  p.gF1 = b.take((int64_t)s.T * s.F * s.E);
  p.ytmp = b.take(TH);
  if (s.pair) {
    const size_t n = (size_t)(s.group - 1) * s.L;
    p.kdy.resize(n); p.kdx2.resize(n); p.kdqkv.resize(n);
    for (size_t i = 0; i < n; ++i) { p.kdy[i] = b.take(TH); p.kdx2[i] = b.take(TH); p.kdqkv[i] = b.take(3 * TH); }
    // scratch for the four weight-gradient products of a full group (smaller groups need less)
    auto need = [&](int M, int N, int batch) {
      Gemm g;
      g.M = M; g.N = N; g.K = s.group * s.T; g.transA = 1; g.c_f32_accum = 1; g.batch = batch; g.nx = s.group - 1; g.kseg = s.T;
      int64_t most = 0;
      for (int nd = 2; nd <= s.group; ++nd) {              // a group closed early has fewer parts
        g.nx = nd - 1; g.K = nd * s.T;
        most = std::max(most, gemm_mfma_ws_bytes(g));
      }
      return most;
    };
    const bool gpt = s.arch == STAGE_ARCH_GPT;
    p.kcut_bytes = std::max(std::max(need(s.F, s.H, 1), gpt ? need(s.H, s.F, 1) : need(s.H, s.F, 2)),
                            std::max(need(s.H, s.H, 1), gpt ? need(s.H, 3 * s.H, 1) : need(s.H, s.H, 3)));
    if (s.bf && p.kcut_bytes) p.kcut = b.take(p.kcut_bytes);
    else p.kcut_bytes = 0;
  }
  p.delta = b.take<float>(4ll * s.mb * s.nh * s.S);
  p.lossdump = b.take<float>(256);
  p.rope = s.arch == STAGE_ARCH_LLAMA ? b.take<float2>(8ll * s.S * (s.d / 2)) : nullptr;
  p.nblk = s.T < MAX_NBLK ? s.T : MAX_NBLK;
  p.partial_floats = (int64_t)p.nblk * (vector_widths_per_layer(s) * s.L + (s.head ? s.H : 0));
  p.partials = b.take<float>(4 * p.partial_floats);
  p.njobs_cap = s.L * 8 + 1;
  p.jobs = b.take<ReduceJob>((int64_t)sizeof(ReduceJob) * p.njobs_cap);
  p.total = ((b.off + 255) & ~(int64_t)255) + (scratch_base ? act_end : 0);
  p.scratch_bytes = p.total - p.act_bytes;
}

void memory_of(const stage_config& c, const Plan& p, stage_memory& m) {
  const Shape s = shape_of(c);
  const int64_t P = count_params(c), sh = c.shard_end - c.shard_begin;
  m.params = P * s.E;
  m.grads = P * 4;
  m.optim = sh * 8 + (s.bf ? sh * 4 : 0);   // m, v (+ fp32 master of the shard)
  m.activations = p.act_bytes;
  m.scratch = p.scratch_bytes;
  m.workspace = p.total;
  m.host_stash = p.host_stash_bytes;
}

// ---- profiling -------------------------------------------------------------------------------
struct ProfRec { int cls; hipEvent_t a, b; double flops, bytes; };

}  // namespace

struct stage {
  stage_config cfg;
  Shape sh;
  hipStream_t st;
  char* params; float *master, *grad, *m, *v;
  std::vector<Seg> layout;
  Plan plan;
  std::vector<int> slot;     // 0 empty, 1 forwarded, 2 backward done (waiting for accumulate)
  int pending = -1;          // slot whose backward waits for stage_accumulate
  int outstanding = 0, accumulated = 0;
  std::vector<int> deferred; // pair_wgrad: slots whose weight-gradient products wait for a later backward (set i = deferred[i])
  int* overflow = nullptr;   // device flag of loss-scaled training (stage_set_overflow_flag), or NULL
  std::vector<ReduceJob> jobs_host;
  int njobs = 0, max_job_width = 0;
  std::string err;
  // offload_acts: boundary activations in pinned host memory, two device slots, one copy stream
  struct DevSlot {
    int owner = -1;            // microbatch whose boundary activations the slot holds (valid or being loaded)
    bool loaded = false;       // the slot's content arrived by a host-to-device copy (readers wait for copy_done)
    bool copied = false, computed = false;   // the events below have been recorded at least once
    hipEvent_t copy_done = nullptr;      // copy stream: last copy from or into the slot has finished
    hipEvent_t compute_done = nullptr;   // stage stream: last forward or backward that used the slot has finished
    int64_t tick = 0;          // last use, for the choice of a victim
  };
  char* host_stash = nullptr;
  hipStream_t copy_st = nullptr;
  DevSlot dslot[2];
  std::vector<int> where;      // per microbatch: device slot that holds its boundary activations, or -1
  int64_t clock = 0;
  // profiling
  bool prof = false;
  std::vector<std::string> cls_names;
  std::vector<ProfRec> recs;
  std::vector<hipEvent_t> ev_pool;
  size_t ev_used = 0;

  int64_t seg_off(const std::string& n) const {
    for (auto& s : layout) if (s.name == n) return s.off;
    return -1;
  }
  char* P(int64_t off) const { return params + off * sh.E; }
  float* G(int64_t off) const { return grad + off; }
};

namespace {

int fail(stage_t* s, int code, const std::string& msg) { if (s) s->err = msg; else g_err = msg; return code; }

int cls_id(stage_t* s, const char* name) {
  for (size_t i = 0; i < s->cls_names.size(); ++i) if (s->cls_names[i] == name) return (int)i;
  s->cls_names.push_back(name);
  return (int)s->cls_names.size() - 1;
}
hipEvent_t next_event(stage_t* s) {
  if (s->ev_used == s->ev_pool.size()) { hipEvent_t e = nullptr; (void)hipEventCreate(&e); s->ev_pool.push_back(e); }
  return s->ev_pool[s->ev_used++];
}

// Runs one launcher on a stream, optionally bracketed by events; returns false (and sets the error) on failure.
template <typename F> bool run_on(stage_t* s, hipStream_t st, const char* cls, double flops, double bytes, F&& f) {
  hipEvent_t a = nullptr, b = nullptr;
  if (s->prof) { a = next_event(s); b = next_event(s); (void)hipEventRecord(a, st); }
  const hipError_t e = f();
  if (s->prof) { (void)hipEventRecord(b, st); s->recs.push_back({cls_id(s, cls), a, b, flops, bytes}); }
  if (e != hipSuccess) { s->err = std::string(cls) + ": " + hipGetErrorString(e); return false; }
  return true;
}
template <typename F> bool run(stage_t* s, const char* cls, double flops, double bytes, F&& f) {
  return run_on(s, s->st, cls, flops, bytes, f);
}

// ---- offload_acts: the device slots and the copies between them and the host stash ------------------
// Ordering rules.  The copy stream is in order, so a load of a microbatch always follows its store.  Before a
// copy touches a device slot the copy stream waits for compute_done of that slot (recorded on the stage's
// stream after every forward or backward that used it); before the stage's stream writes a slot, or reads one
// that was filled by a load, it waits for the slot's copy_done.
bool hip_ok(stage_t* s, hipError_t e, const char* what) {
  if (e == hipSuccess) return true;
  s->err = std::string(what) + ": " + hipGetErrorString(e);
  return false;
}

void evict(stage_t* s, int k) {
  stage::DevSlot& d = s->dslot[k];
  if (d.owner >= 0 && s->where[d.owner] == k) s->where[d.owner] = -1;
  d.owner = -1;
}

// A slot whose microbatch is no longer waiting for its backward first, else the least recently used one (its
// microbatch stays valid on the host).
int pick_slot(stage_t* s) {
  int best = -1;
  for (int k = 0; k < s->plan.dev_slots; ++k) {
    const stage::DevSlot& d = s->dslot[k];
    if (d.owner < 0 || s->slot[d.owner] != 1) return k;
    if (best < 0 || d.tick < s->dslot[best].tick) best = k;
  }
  return best;
}

bool mark_computed(stage_t* s, int k) {
  stage::DevSlot& d = s->dslot[k];
  d.computed = true;
  return hip_ok(s, hipEventRecord(d.compute_done, s->st), "offload: event record");
}

// The copies are left to the runtime's copy path (hipMemcpyAsync on the copy stream).  A copy kernel of this
// library reached the full link rate (55 GB/s each way) but cost 13-19 % of the step: the GEMM grids fill the
// 256 compute units exactly, so every unit held by a resident copy workgroup adds a round to each of them.
// After forward(mb) wrote slot k: copy it to the host.
bool offload_store(stage_t* s, int k, int mb) {
  stage::DevSlot& d = s->dslot[k];
  if (!mark_computed(s, k)) return false;
  if (!hip_ok(s, hipStreamWaitEvent(s->copy_st, d.compute_done, 0), "offload: stream wait")) return false;
  const int64_t n = s->plan.slot_bytes;
  if (!run_on(s, s->copy_st, "offload_d2h", 0, (double)n, [&] {
        return hipMemcpyAsync(s->host_stash + (int64_t)mb * n, s->plan.stash[(size_t)k * s->sh.L], n, hipMemcpyDeviceToHost,
                              s->copy_st); }))
    return false;
  d.copied = true;
  return hip_ok(s, hipEventRecord(d.copy_done, s->copy_st), "offload: event record");
}

// Brings microbatch mb from the host into slot k (whose previous content is given up).
bool offload_load(stage_t* s, int k, int mb) {
  evict(s, k);
  stage::DevSlot& d = s->dslot[k];
  if (d.computed && !hip_ok(s, hipStreamWaitEvent(s->copy_st, d.compute_done, 0), "offload: stream wait")) return false;
  const int64_t n = s->plan.slot_bytes;
  if (!run_on(s, s->copy_st, "offload_h2d", 0, (double)n, [&] {
        return hipMemcpyAsync(s->plan.stash[(size_t)k * s->sh.L], s->host_stash + (int64_t)mb * n, n, hipMemcpyHostToDevice,
                              s->copy_st); }))
    return false;
  d.owner = mb; d.loaded = true; d.copied = true; d.tick = ++s->clock;
  s->where[mb] = k;
  return hip_ok(s, hipEventRecord(d.copy_done, s->copy_st), "offload: event record");
}

DType dt_of(const stage_t* s) { return s->sh.dtype == STAGE_DTYPE_F16 ? F16 : s->sh.bf ? BF16 : F32; }

bool do_gemm(stage_t* s, const Gemm& g) {
  const int impl = gemm_select(dt_of(s), g, GEMM_AUTO);
  static const char* names[2][4] = {{"gemm_simple_nn", "gemm_simple_nt", "gemm_simple_tn", "gemm_simple_tt"},
                                    {"gemm_mfma_nn", "gemm_mfma_nt", "gemm_mfma_tn", "gemm_mfma_tt"}};
  const bool mfma = impl == GEMM_MFMA || gemm_splits(dt_of(s), g);
  // the products that apply the gated unit in their store are kernels of their own and are timed as such
  const char* cls = mfma && g.glu == 1 ? "gemm_mfma_nn_glu" : mfma && g.glu == 2 ? "gemm_mfma_nt_glu" : names[mfma][g.transA * 2 + g.transB];
  const double flops = 2.0 * g.M * g.N * g.K * (g.glu == 1 ? 2 : g.batch);
  return run(s, cls, flops, 0.0, [&] { return gemm(s->st, dt_of(s), g, GEMM_AUTO); });
}

// ---- forward of one layer ---------------------------------------------------------------------
// x_in -> y (y may be NULL: recompute pass, the output is not needed).
bool layer_forward(stage_t* s, int l, const char* x_in, LayerActs& A, char* y) {
  const Shape& h = s->sh;
  const DType dt = dt_of(s);
  const int T = h.T, H = h.H, F = h.F;
  const std::string p = "L" + std::to_string(l) + ".";
  const double thb = (double)T * H * h.E;
  const bool gpt = h.arch == STAGE_ARCH_GPT;
  auto W = [&](const char* n) { return s->P(s->seg_off(p + n)); };

  if (!run(s, "norm_fwd", 0, 2 * thb, [&] {
        return gpt ? norm_fwd(s->st, dt, 0, T, H, x_in, W("ln1.g"), W("ln1.b"), s->cfg.norm_eps, A.n1, A.rstd1, A.mean1)
                   : norm_fwd(s->st, dt, 1, T, H, x_in, W("rms1.g"), nullptr, s->cfg.norm_eps, A.n1, A.rstd1, nullptr); }))
    return false;
  Gemm g;
  g.M = T; g.K = H; g.A = A.n1; g.lda = H; g.C = A.qkv; g.ldc = 3 * H;
  if (gpt) { g.N = 3 * H; g.B = W("Wqkv"); g.ldb = 3 * H; g.bias = W("bqkv"); }
  else {   // Q and K leave the projection already rotated
    g.N = H; g.B = W("Wq"); g.ldb = H; g.batch = 3; g.sB = (int64_t)H * H; g.sC = H;
    g.rope = s->plan.rope; g.rope_S = h.S; g.rope_d = h.d; g.rope_batches = 2;
  }
  if (!do_gemm(s, g)) return false;
  const double attn_flops = 4.0 * h.mb * h.nh * (double)h.S * (h.S + 1) / 2 * h.d;
  if (!run(s, attn_select(dt, h.S, h.d, 0) == ATTN_MFMA ? "attn_fwd_mfma" : "attn_fwd_simple", attn_flops, 0, [&] {
        return attn_fwd(s->st, dt, h.mb, h.S, h.nh, h.d, A.qkv, A.qkv + (int64_t)H * h.E, A.qkv + 2ll * H * h.E, 3 * H,
                        A.o, H, A.lse, ATTN_AUTO); }))
    return false;
  g = Gemm();
  g.M = T; g.N = H; g.K = H; g.A = A.o; g.lda = H; g.B = W("Wo"); g.ldb = H; g.C = A.x2; g.ldc = H;
  g.resid = x_in; g.ldr = H; if (gpt) g.bias = W("bo");
  if (!do_gemm(s, g)) return false;
  if (!run(s, "norm_fwd", 0, 2 * thb, [&] {
        return gpt ? norm_fwd(s->st, dt, 0, T, H, A.x2, W("ln2.g"), W("ln2.b"), s->cfg.norm_eps, A.n2, A.rstd2, A.mean2)
                   : norm_fwd(s->st, dt, 1, T, H, A.x2, W("rms2.g"), nullptr, s->cfg.norm_eps, A.n2, A.rstd2, nullptr); }))
    return false;
  g = Gemm();
  g.M = T; g.K = H; g.A = A.n2; g.lda = H; g.N = F; g.ldb = F;
  if (gpt) { g.B = W("W1"); g.C = A.ff; g.ldc = F; g.bias = W("b1"); }
  else {   // gate and up projections in one product whose store applies the gated unit: ff = [gate | up], a = silu(gate) * up
    g.B = W("Wg"); g.sB = (int64_t)H * F; g.C = A.a; g.ldc = F; g.glu = 1; g.gu = A.ff; g.gu_ld = 2 * F; g.gu_up = F;
  }
  if (!do_gemm(s, g)) return false;
  const double tfb = (double)T * F * h.E;
  if (gpt && !run(s, "activation", 0, 2 * tfb, [&] { return gelu_fwd(s->st, dt, (int64_t)T * F, A.ff, A.a); })) return false;
  if (!y) return true;
  g = Gemm();
  g.M = T; g.N = H; g.K = F; g.A = A.a; g.lda = F; g.B = gpt ? W("W2") : W("Wd"); g.ldb = H; g.C = y; g.ldc = H;
  g.resid = A.x2; g.ldr = H; if (gpt) g.bias = W("b2");
  return do_gemm(s, g);
}

// Partials of the vector parameters: segment -> float[nblk, width] inside plan.partials.
float* partial_of(stage_t* s, const std::string& name) {
  for (int i = 0; i < s->njobs; ++i)
    if (s->jobs_host[i].dst == s->G(s->seg_off(name))) return const_cast<float*>(s->jobs_host[i].part);
  return nullptr;
}

bool colsum(stage_t* s, const std::string& seg, int N, const void* a, int64_t lda, const void* x, const float* rstd,
            const float* mean) {
  const Shape& h = s->sh;
  float* part = partial_of(s, seg);
  return run(s, "colsum", 0, (double)h.T * N * h.E * (x ? 2 : 1), [&] {
    return colsum_partial(s->st, dt_of(s), h.T, N, a, lda, x, N, rstd, mean, part, s->plan.nblk); });
}

// ---- backward of one layer ----------------------------------------------------------------------
// dy -> dx.  dy and dx are distinct [T,H] buffers; tmp is a third one (holds dx2).
// Weight-gradient products of a layer: done now (mode 0), left for later (1: this microbatch's operands
// stay where they are), or done for this microbatch and a deferred one in one product (2).
struct WgradPlan {
  int mode = 0;                                           // 0 plain, 1 leave the products to a later backward, 2 multiply for nx more
  int nx = 0;
  const LayerActs* Ax[GEMM_MAX_PARTS - 1] = {};           // mode 2: the deferred microbatches' activations of this layer ...
  const char *dy_x[GEMM_MAX_PARTS - 1] = {}, *dx2_x[GEMM_MAX_PARTS - 1] = {}, *dqkv_x[GEMM_MAX_PARTS - 1] = {};   // ... and their dy, dx2, dqkv
};

bool layer_backward(stage_t* s, int l, const char* x_in, LayerActs& A, const char* dy, char* tmp, char* dx, char* gqkv,
                    const WgradPlan& wg) {
  const Shape& h = s->sh;
  const DType dt = dt_of(s);
  const int T = h.T, H = h.H, F = h.F;
  const std::string p = "L" + std::to_string(l) + ".";
  const bool gpt = h.arch == STAGE_ARCH_GPT;
  const double thb = (double)T * H * h.E, tfb = (double)T * F * h.E;
  Plan& pl = s->plan;
  auto W = [&](const char* n) { return s->P(s->seg_off(p + n)); };
  auto GW = [&](const char* n) { return s->G(s->seg_off(p + n)); };
  Gemm g;
  // dW += X^T dY over this microbatch's tokens, and over the deferred microbatches' too when there are any:
  // xsel picks the activation of a deferred microbatch, dsel its gradient operand
  auto wgrad = [&](Gemm w, char* LayerActs::*xsel, auto dsel) {
    if (wg.mode == 1) return true;
    if (wg.mode == 2) {
      w.nx = wg.nx; w.kseg = T; w.K = (wg.nx + 1) * T;
      for (int i = 0; i < wg.nx; ++i) { w.Ax[i] = wg.Ax[i]->*xsel; w.Bx[i] = dsel(i); }
      w.ws = pl.kcut; w.ws_bytes = pl.kcut_bytes;
    }
    return do_gemm(s, w);
  };

  // FFN down projection: da = dy Wd^T ; dWd += a^T dy
  g.M = T; g.N = F; g.K = H; g.A = dy; g.lda = H; g.B = gpt ? W("W2") : W("Wd"); g.ldb = H; g.transB = 1;
  g.C = pl.gF1; g.ldc = F;
  // Llama: the store turns (gate, up), saved in ff, into (dgate, dup) in place; da itself is not kept
  if (!gpt) { g.glu = 2; g.gu = A.ff; g.gu_ld = 2 * F; g.gu_up = F; }
  if (!do_gemm(s, g)) return false;
  g = Gemm();
  g.M = F; g.N = H; g.K = T; g.A = A.a; g.lda = F; g.transA = 1; g.B = dy; g.ldb = H;
  g.C = gpt ? GW("W2") : GW("Wd"); g.ldc = H; g.c_f32_accum = 1;
  if (!wgrad(g, &LayerActs::a, [&](int i) { return wg.dy_x[i]; })) return false;
  if (gpt && !colsum(s, p + "b2", H, dy, H, nullptr, nullptr, nullptr)) return false;

  // GELU backward, in place over the saved pre-activations
  if (gpt && !run(s, "activation", 0, 3 * tfb, [&] { return gelu_bwd(s->st, dt, (int64_t)T * F, A.ff, pl.gF1, A.ff); }))
    return false;
  const char* dff = A.ff;   // dz [T,F] or [dgate | dup] [T,2F]

  // FFN up projection(s): dn2 = dff W^T ; dW += n2^T dff
  g = Gemm();
  g.M = T; g.N = H; g.A = dff; g.transB = 1; g.C = pl.gN; g.ldc = H; g.ldb = F;
  if (gpt) { g.K = F; g.lda = F; g.B = W("W1"); }
  else { g.K = 2 * F; g.lda = 2 * F; g.B = W("Wg"); g.kseg = F; g.segB = (int64_t)H * F; }
  if (!do_gemm(s, g)) return false;
  g = Gemm();
  g.M = H; g.N = F; g.K = T; g.A = A.n2; g.lda = H; g.transA = 1; g.B = dff; g.c_f32_accum = 1; g.ldc = F;
  if (gpt) { g.ldb = F; g.C = GW("W1"); }
  else { g.ldb = 2 * F; g.C = GW("Wg"); g.batch = 2; g.sB = F; g.sC = (int64_t)H * F; }
  if (!wgrad(g, &LayerActs::n2, [&](int i) { return (const char*)wg.Ax[i]->ff; })) return false;
  if (gpt && !colsum(s, p + "b1", F, dff, F, nullptr, nullptr, nullptr)) return false;

  // second norm: gain (and bias) partials, dx2 = dy + norm'(x2)^T dn2
  if (!run(s, "norm_bwd", 0, 4 * thb, [&] {
        return norm_bwd_partials(s->st, dt, gpt ? 0 : 1, T, H, pl.gN, A.x2, gpt ? W("ln2.g") : W("rms2.g"), A.rstd2,
                                 A.mean2, dy, tmp, partial_of(s, p + (gpt ? "ln2.g" : "rms2.g")),
                                 gpt ? partial_of(s, p + "ln2.b") : nullptr, s->plan.nblk); }))
    return false;

  // attention output projection: do = dx2 Wo^T ; dWo += o^T dx2
  g = Gemm();
  g.M = T; g.N = H; g.K = H; g.A = tmp; g.lda = H; g.B = W("Wo"); g.ldb = H; g.transB = 1; g.C = pl.gO; g.ldc = H;
  if (!do_gemm(s, g)) return false;
  g = Gemm();
  g.M = H; g.N = H; g.K = T; g.A = A.o; g.lda = H; g.transA = 1; g.B = tmp; g.ldb = H; g.C = GW("Wo"); g.ldc = H;
  g.c_f32_accum = 1;
  if (!wgrad(g, &LayerActs::o, [&](int i) { return wg.dx2_x[i]; })) return false;
  if (gpt && !colsum(s, p + "bo", H, tmp, H, nullptr, nullptr, nullptr)) return false;

  // attention backward (+ inverse rotation of dq, dk)
  // algorithmic work: dV, dP, dQ, dK over the causal half (recomputing the scores is not counted)
  const double attn_flops = 8.0 * h.mb * h.nh * (double)h.S * (h.S + 1) / 2 * h.d;
  const int64_t HE = (int64_t)H * h.E;
  if (!run(s, attn_select(dt, h.S, h.d, 0) == ATTN_MFMA ? "attn_bwd_mfma" : "attn_bwd_simple", attn_flops, 0, [&] {
        return attn_bwd(s->st, dt, h.mb, h.S, h.nh, h.d, A.qkv, A.qkv + HE, A.qkv + 2 * HE, 3 * H, A.o, pl.gO, H, A.lse,
                        pl.delta, gqkv, gqkv + HE, gqkv + 2 * HE, 3 * H, gpt ? nullptr : pl.rope, ATTN_AUTO); }))
    return false;

  // QKV projection: dn1 = dqkv [Wq|Wk|Wv]^T ; dW += n1^T dqkv
  g = Gemm();
  g.M = T; g.N = H; g.K = 3 * H; g.A = gqkv; g.lda = 3 * H; g.transB = 1; g.C = pl.gN; g.ldc = H;
  if (gpt) { g.B = W("Wqkv"); g.ldb = 3 * H; }
  else { g.B = W("Wq"); g.ldb = H; g.kseg = H; g.segB = (int64_t)H * H; }
  if (!do_gemm(s, g)) return false;
  g = Gemm();
  g.M = H; g.K = T; g.A = A.n1; g.lda = H; g.transA = 1; g.B = gqkv; g.ldb = 3 * H; g.c_f32_accum = 1;
  if (gpt) { g.N = 3 * H; g.C = GW("Wqkv"); g.ldc = 3 * H; }
  else { g.N = H; g.C = GW("Wq"); g.ldc = H; g.batch = 3; g.sB = H; g.sC = (int64_t)H * H; }
  if (!wgrad(g, &LayerActs::n1, [&](int i) { return wg.dqkv_x[i]; })) return false;
  if (gpt && !colsum(s, p + "bqkv", 3 * H, gqkv, 3 * H, nullptr, nullptr, nullptr)) return false;

  // first norm: dx = dx2 + norm'(x)^T dn1
  return run(s, "norm_bwd", 0, 4 * thb, [&] {
    return norm_bwd_partials(s->st, dt, gpt ? 0 : 1, T, H, pl.gN, x_in, gpt ? W("ln1.g") : W("rms1.g"), A.rstd1, A.mean1,
                             tmp, dx, partial_of(s, p + (gpt ? "ln1.g" : "rms1.g")),
                             gpt ? partial_of(s, p + "ln1.b") : nullptr, s->plan.nblk); });
}

bool head_forward(stage_t* s, const char* y, HeadActs& A, const int32_t* targets, float* loss_out) {
  const Shape& h = s->sh;
  const DType dt = dt_of(s);
  if (!run(s, "norm_fwd", 0, 2.0 * h.T * h.H * h.E, [&] {
        return norm_fwd(s->st, dt, 1, h.T, h.H, y, s->P(s->seg_off("final_norm.g")), nullptr, s->cfg.norm_eps, A.nf, A.rstd, nullptr); }))
    return false;
  Gemm g;
  g.M = h.T; g.N = h.V; g.K = h.H; g.A = A.nf; g.lda = h.H; g.B = s->P(s->seg_off("head.Wh")); g.ldb = h.V;
  g.C = A.logits; g.ldc = h.V;
  if (!do_gemm(s, g)) return false;
  return run(s, "cross_entropy", 0, (double)h.T * h.V * h.E, [&] {
    return ce_fwd(s->st, dt, h.T, h.V, A.logits, h.V, targets, A.lse, A.rowloss, loss_out); });
}

bool head_backward(stage_t* s, const char* y, HeadActs& A, const int32_t* targets, float loss_scale, char* dcur) {
  const Shape& h = s->sh;
  const DType dt = dt_of(s);
  Plan& pl = s->plan;
  if (!run(s, "cross_entropy", 0, 2.0 * h.T * h.V * h.E, [&] {
        return ce_bwd(s->st, dt, h.T, h.V, A.logits, h.V, targets, A.lse, loss_scale / (float)h.T); }))
    return false;
  Gemm g;
  g.M = h.H; g.N = h.V; g.K = h.T; g.A = A.nf; g.lda = h.H; g.transA = 1; g.B = A.logits; g.ldb = h.V;
  g.C = s->G(s->seg_off("head.Wh")); g.ldc = h.V; g.c_f32_accum = 1;
  if (!do_gemm(s, g)) return false;
  g = Gemm();
  g.M = h.T; g.N = h.H; g.K = h.V; g.A = A.logits; g.lda = h.V; g.B = s->P(s->seg_off("head.Wh")); g.ldb = h.V;
  g.transB = 1; g.C = pl.gN; g.ldc = h.H;
  if (!do_gemm(s, g)) return false;
  return run(s, "norm_bwd", 0, 3.0 * h.T * h.H * h.E, [&] {
    return norm_bwd_partials(s->st, dt, 1, h.T, h.H, pl.gN, y, s->P(s->seg_off("final_norm.g")), A.rstd, nullptr, nullptr,
                             dcur, partial_of(s, "final_norm.g"), nullptr, s->plan.nblk); });
}

bool check_slot(stage_t* s, int mb) { return mb >= 0 && mb < s->sh.M; }

// The weight-gradient products of the deferred microbatches on their own (a slot is about to be reused, or
// the step ends): one multi-part product per weight over all of them.
bool flush_deferred(stage_t* s) {
  const int nd = (int)s->deferred.size();
  if (nd == 0) return true;
  const Shape& h = s->sh;
  Plan& pl = s->plan;
  const int T = h.T, H = h.H, F = h.F;
  const bool gpt = h.arch == STAGE_ARCH_GPT;
  for (int l = h.L - 1; l >= 0; --l) {
    auto acts = [&](int i) -> const LayerActs& { return pl.acts[(size_t)s->deferred[i] * h.L + l]; };
    const std::string p = "L" + std::to_string(l) + ".";
    auto GW = [&](const char* n) { return s->G(s->seg_off(p + n)); };
    auto parts = [&](Gemm& g, char* LayerActs::*xsel, auto dsel) {   // part 0 = first deferred, the others follow
      g.A = acts(0).*xsel; g.B = dsel(0);
      g.K = nd * T;
      if (nd > 1) { g.nx = nd - 1; g.kseg = T; g.ws = pl.kcut; g.ws_bytes = pl.kcut_bytes; }
      for (int i = 1; i < nd; ++i) { g.Ax[i - 1] = acts(i).*xsel; g.Bx[i - 1] = dsel(i); }
    };
    Gemm g;
    g.M = F; g.N = H; g.lda = F; g.transA = 1; g.ldb = H;
    g.C = gpt ? GW("W2") : GW("Wd"); g.ldc = H; g.c_f32_accum = 1;
    parts(g, &LayerActs::a, [&](int i) { return (const char*)pl.kdy[(size_t)i * h.L + l]; });
    if (!do_gemm(s, g)) return false;
    g = Gemm();
    g.M = H; g.N = F; g.lda = H; g.transA = 1; g.c_f32_accum = 1; g.ldc = F;
    if (gpt) { g.ldb = F; g.C = GW("W1"); }
    else { g.ldb = 2 * F; g.C = GW("Wg"); g.batch = 2; g.sB = F; g.sC = (int64_t)H * F; }
    parts(g, &LayerActs::n2, [&](int i) { return (const char*)acts(i).ff; });
    if (!do_gemm(s, g)) return false;
    g = Gemm();
    g.M = H; g.N = H; g.lda = H; g.transA = 1; g.ldb = H; g.C = GW("Wo"); g.ldc = H;
    g.c_f32_accum = 1;
    parts(g, &LayerActs::o, [&](int i) { return (const char*)pl.kdx2[(size_t)i * h.L + l]; });
    if (!do_gemm(s, g)) return false;
    g = Gemm();
    g.M = H; g.lda = H; g.transA = 1; g.ldb = 3 * H; g.c_f32_accum = 1;
    if (gpt) { g.N = 3 * H; g.C = GW("Wqkv"); g.ldc = 3 * H; }
    else { g.N = H; g.C = GW("Wq"); g.ldc = H; g.batch = 3; g.sB = H; g.sC = (int64_t)H * H; }
    parts(g, &LayerActs::n1, [&](int i) { return (const char*)pl.kdqkv[(size_t)i * h.L + l]; });
    if (!do_gemm(s, g)) return false;
  }
  s->deferred.clear();
  return true;
}

}  // namespace

extern "C" {

int stage_query(const stage_config* cfg, int64_t* n_params, stage_memory* mem, int32_t* n_segments) {
  std::string err;
  const int rc = validate(cfg, err);
  if (rc != STAGE_OK) return fail(nullptr, rc, err);
  Plan p;
  make_plan(*cfg, nullptr, p);
  stage_memory m;
  memory_of(*cfg, p, m);
  if (n_params) *n_params = count_params(*cfg);
  if (mem) *mem = m;
  if (n_segments) *n_segments = (int32_t)make_layout(*cfg).size();
  if (cfg->act_budget_bytes > 0 && m.activations + m.scratch > cfg->act_budget_bytes)
    return fail(nullptr, STAGE_ERR_BUDGET, "activations + scratch = " + std::to_string(m.activations + m.scratch) +
                                               " bytes exceed act_budget_bytes = " + std::to_string(cfg->act_budget_bytes));
  return STAGE_OK;
}

int stage_layout(const stage_config* cfg, stage_segment* out, int32_t n_segments) {
  std::string err;
  const int rc = validate(cfg, err);
  if (rc != STAGE_OK) return fail(nullptr, rc, err);
  const auto lay = make_layout(*cfg);
  if (!out || n_segments != (int32_t)lay.size()) return fail(nullptr, STAGE_ERR_ARG, "n_segments does not match stage_query");
  for (size_t i = 0; i < lay.size(); ++i) {
    std::memset(out[i].name, 0, sizeof(out[i].name));
    std::strncpy(out[i].name, lay[i].name.c_str(), sizeof(out[i].name) - 1);
    out[i].offset = lay[i].off; out[i].rows = lay[i].rows; out[i].cols = lay[i].cols;
  }
  return STAGE_OK;
}

int stage_init(const stage_config* cfg, void* hip_stream, void* params, float* master, float* grad_acc, float* adam_m,
               float* adam_v, void* workspace, int64_t workspace_bytes, stage_t** out) {
  return stage_init_split(cfg, hip_stream, params, master, grad_acc, adam_m, adam_v, workspace, workspace_bytes, nullptr, 0, out);
}

int stage_init_split(const stage_config* cfg, void* hip_stream, void* params, float* master, float* grad_acc, float* adam_m,
                     float* adam_v, void* workspace, int64_t workspace_bytes, void* scratch, int64_t scratch_bytes,
                     stage_t** out) {
  if (out) *out = nullptr;
  if (!out) return fail(nullptr, STAGE_ERR_ARG, "out is NULL");
  stage_memory mem;
  const int rc = stage_query(cfg, nullptr, &mem, nullptr);
  if (rc != STAGE_OK) return rc;
  const int64_t sh = cfg->shard_end - cfg->shard_begin;
  if (!params || !grad_acc) return fail(nullptr, STAGE_ERR_ARG, "params and grad_acc must not be NULL");
  if (sh > 0 && (!adam_m || !adam_v)) return fail(nullptr, STAGE_ERR_ARG, "adam_m and adam_v must not be NULL");
  if (cfg->dtype != STAGE_DTYPE_F32 && sh > 0 && !master) return fail(nullptr, STAGE_ERR_ARG, "master must not be NULL for dtypes 1 and 2");
  if (cfg->dtype == STAGE_DTYPE_F32 && master) return fail(nullptr, STAGE_ERR_ARG, "master must be NULL for dtype 0");
  if (((uintptr_t)params | (uintptr_t)grad_acc | (uintptr_t)master | (uintptr_t)adam_m | (uintptr_t)adam_v) & 15)
    return fail(nullptr, STAGE_ERR_ARG, "params, master, grad_acc, adam_m, adam_v must be 16-byte aligned");
  if (!workspace || ((uintptr_t)workspace & 255)) return fail(nullptr, STAGE_ERR_WORKSPACE, "workspace is NULL or not 256-byte aligned");
  const int64_t act_part = (mem.activations + 255) & ~(int64_t)255;   // with a scratch buffer of its own: the two parts
  const int64_t need_ws = scratch ? act_part : mem.workspace, need_scratch = mem.workspace - act_part;
  if (workspace_bytes < need_ws)
    return fail(nullptr, STAGE_ERR_WORKSPACE, "workspace has " + std::to_string(workspace_bytes) + " bytes, " +
                                                  std::to_string(need_ws) + " needed");
  if (scratch && (((uintptr_t)scratch & 255) || scratch_bytes < need_scratch))
    return fail(nullptr, STAGE_ERR_WORKSPACE, "scratch is not 256-byte aligned or has fewer than " + std::to_string(need_scratch) + " bytes");
  stage_t* s = new stage();
  s->cfg = *cfg;
  s->sh = shape_of(*cfg);
  s->st = (hipStream_t)hip_stream;
  s->params = (char*)params; s->master = master; s->grad = grad_acc; s->m = adam_m; s->v = adam_v;
  s->layout = make_layout(*cfg);
  make_plan(*cfg, (char*)workspace, s->plan, (char*)scratch);
  s->slot.assign(s->sh.M, 0);
  s->where.assign(s->sh.M, -1);

  // reduction jobs of the vector parameters, partial buffers carved in layout order
  float* pp = s->plan.partials;
  for (auto& seg : s->layout) {
    if (seg.rows != 1) continue;
    ReduceJob j;
    j.part = pp; j.dst = s->G(seg.off); j.nblk = s->plan.nblk; j.width = (int)seg.cols;
    pp += (int64_t)s->plan.nblk * seg.cols;
    s->jobs_host.push_back(j);
    if ((int)seg.cols > s->max_job_width) s->max_job_width = (int)seg.cols;
  }
  s->njobs = (int)s->jobs_host.size();
  hipError_t e = hipSuccess;
  if (s->njobs)
    e = hipMemcpyAsync(s->plan.jobs, s->jobs_host.data(), sizeof(ReduceJob) * s->njobs, hipMemcpyHostToDevice, s->st);
  if (e == hipSuccess && s->plan.rope) e = rope_table(s->st, s->sh.S, s->sh.d, cfg->rope_base, s->plan.rope);
  if (e != hipSuccess) {
    const std::string msg = std::string("stage_init: ") + hipGetErrorString(e);
    delete s;
    return fail(nullptr, STAGE_ERR_DEVICE, msg);
  }
  *out = s;
  return STAGE_OK;
}

int stage_attach_host_stash(stage_t* s, void* host_pinned, int64_t bytes) {
  if (!s) return STAGE_ERR_ARG;
  if (!s->sh.offload) return fail(s, STAGE_ERR_ARG, "the stage was not configured with offload_acts = 1");
  if (s->host_stash) return fail(s, STAGE_ERR_STATE, "a host buffer is already attached");
  if (!host_pinned) return fail(s, STAGE_ERR_ARG, "host_pinned is NULL");
  if (bytes < s->plan.host_stash_bytes)
    return fail(s, STAGE_ERR_ARG, "host buffer has " + std::to_string(bytes) + " bytes, " +
                                      std::to_string(s->plan.host_stash_bytes) + " needed");
  hipPointerAttribute_t at;
  if (hipPointerGetAttributes(&at, host_pinned) != hipSuccess) {
    (void)hipGetLastError();   // the query of an unknown pointer leaves an error behind
    return fail(s, STAGE_ERR_ARG, "host buffer is not page-locked (allocate it with hipHostMalloc)");
  }
  if (at.type != hipMemoryTypeHost)
    return fail(s, STAGE_ERR_ARG, "host buffer is not page-locked host memory (allocate it with hipHostMalloc)");
  hipError_t e = hipStreamCreateWithFlags(&s->copy_st, hipStreamNonBlocking);   // default priority
  for (int k = 0; k < 2 && e == hipSuccess; ++k) {
    e = hipEventCreateWithFlags(&s->dslot[k].copy_done, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->dslot[k].compute_done, hipEventDisableTiming);
  }
  if (e != hipSuccess) return fail(s, STAGE_ERR_DEVICE, std::string("stage_attach_host_stash: ") + hipGetErrorString(e));
  s->host_stash = (char*)host_pinned;
  return STAGE_OK;
}

int stage_forward(stage_t* s, int32_t mb, const void* x_or_ids, void* y_out, const int32_t* targets, float* loss_out) {
  if (!s) return STAGE_ERR_ARG;
  const Shape& h = s->sh;
  if (!check_slot(s, mb)) return fail(s, STAGE_ERR_ARG, "microbatch slot out of range");
  if (!x_or_ids) return fail(s, STAGE_ERR_ARG, "x_or_ids is NULL");
  if (h.head && (!targets || !loss_out)) return fail(s, STAGE_ERR_ARG, "targets and loss_out are required when has_head");
  if (!h.head && !y_out) return fail(s, STAGE_ERR_ARG, "y_out is NULL");
  if (s->pending >= 0) return fail(s, STAGE_ERR_STATE, "a backward is waiting for stage_accumulate");
  if (s->slot[mb] != 0) return fail(s, STAGE_ERR_STATE, "slot already holds a forward that was not backpropagated");
  for (int d : s->deferred)   // a deferred microbatch's activations are about to be overwritten
    if (d == mb) { if (!flush_deferred(s)) return STAGE_ERR_DEVICE; break; }
  Plan& pl = s->plan;
  const DType dt = dt_of(s);
  const int64_t TH = (int64_t)h.T * h.H * h.E;

  int k = mb;   // index of the microbatch's boundary activations on the device
  if (h.offload) {
    if (!s->host_stash) return fail(s, STAGE_ERR_STATE, "offload_acts = 1 but stage_attach_host_stash was not called");
    if (s->where[mb] >= 0) evict(s, s->where[mb]);   // left over from this slot's previous round
    k = pick_slot(s);
    evict(s, k);
    stage::DevSlot& d = s->dslot[k];
    if (d.copied && !hip_ok(s, hipStreamWaitEvent(s->st, d.copy_done, 0), "offload: stream wait")) return STAGE_ERR_DEVICE;
    d.owner = mb; d.loaded = false; d.tick = ++s->clock;
    s->where[mb] = k;
  }
  auto in_of = [&](int l) { return h.recompute ? pl.stash[(size_t)k * h.L + l] : pl.acts[(size_t)mb * h.L + l].x_in; };
  char* x0 = in_of(0);
  if (h.embed) {
    if (!run(s, "copy", 0, 8.0 * h.T, [&] { return copy_bytes(s->st, pl.ids[mb], x_or_ids, 4ll * h.T); })) return STAGE_ERR_DEVICE;
    if (!run(s, "embed", 0, 2.0 * TH, [&] {
          return embed_fwd(s->st, dt, h.T, h.H, h.V, pl.ids[mb], s->P(s->seg_off("embed.E")), x0); }))
      return STAGE_ERR_DEVICE;
  } else if (!run(s, "copy", 0, 2.0 * TH, [&] { return copy_bytes(s->st, x0, x_or_ids, TH); })) {
    return STAGE_ERR_DEVICE;
  }
  char* final_y = nullptr;
  if (h.head) final_y = h.recompute ? pl.hstash[k] : pl.hacts[mb].y;
  for (int l = 0; l < h.L; ++l) {
    LayerActs& A = h.recompute ? pl.acts[0] : pl.acts[(size_t)mb * h.L + l];
    char* y = l + 1 < h.L ? in_of(l + 1) : (h.head ? final_y : (char*)y_out);
    if (!layer_forward(s, l, in_of(l), A, y)) return STAGE_ERR_DEVICE;
  }
  if (h.head) {
    if (!run(s, "copy", 0, 8.0 * h.T, [&] { return copy_bytes(s->st, pl.targets[mb], targets, 4ll * h.T); })) return STAGE_ERR_DEVICE;
    HeadActs& HA = h.recompute ? pl.hacts[0] : pl.hacts[mb];
    if (!head_forward(s, final_y, HA, pl.targets[mb], loss_out)) return STAGE_ERR_DEVICE;
    if (y_out && !run(s, "copy", 0, 2.0 * TH, [&] { return copy_bytes(s->st, y_out, final_y, TH); })) return STAGE_ERR_DEVICE;
  }
  if (h.offload && !offload_store(s, k, mb)) return STAGE_ERR_DEVICE;
  s->slot[mb] = 1;
  s->outstanding++;
  return STAGE_OK;
}

int stage_backward(stage_t* s, int32_t mb, const void* dy, void* dx_out, float loss_scale) {
  if (!s) return STAGE_ERR_ARG;
  const Shape& h = s->sh;
  if (!check_slot(s, mb)) return fail(s, STAGE_ERR_ARG, "microbatch slot out of range");
  if (!h.head && !dy) return fail(s, STAGE_ERR_ARG, "dy is NULL");
  if (!h.embed && !dx_out) return fail(s, STAGE_ERR_ARG, "dx_out is NULL");
  if (s->pending >= 0) return fail(s, STAGE_ERR_STATE, "the previous backward is waiting for stage_accumulate");
  if (s->slot[mb] != 1) return fail(s, STAGE_ERR_STATE, "slot holds no forward");
  Plan& pl = s->plan;
  const int64_t TH = (int64_t)h.T * h.H * h.E;

  int k = mb;   // index of the microbatch's boundary activations on the device
  if (h.offload) {
    k = s->where[mb];
    if (k < 0) {   // not on the device (any more): load it now, the kernels below wait for it
      k = pick_slot(s);
      if (!offload_load(s, k, mb)) return STAGE_ERR_DEVICE;
    }
    stage::DevSlot& d = s->dslot[k];
    d.tick = ++s->clock;
    if (d.loaded && !hip_ok(s, hipStreamWaitEvent(s->st, d.copy_done, 0), "offload: stream wait")) return STAGE_ERR_DEVICE;
    // the next microbatch of the reverse order travels to the other slot while this one computes
    const int nx = mb - 1;
    if (pl.dev_slots > 1 && nx >= 0 && s->slot[nx] == 1 && s->where[nx] < 0 && !offload_load(s, 1 - k, nx))
      return STAGE_ERR_DEVICE;
  }
  auto in_of = [&](int l) { return h.recompute ? pl.stash[(size_t)k * h.L + l] : pl.acts[(size_t)mb * h.L + l].x_in; };
  // pair_wgrad: a backward with further backwards to come leaves its weight-gradient products to a later one and
  // keeps their dY operands in per-layer buffers; the backward that completes a group of `group` microbatches,
  // or the last outstanding one, multiplies for all of them in one K loop per weight.
  const int nd = (int)s->deferred.size();
  const bool last = s->outstanding == 1;
  const bool fuse = h.pair && nd > 0 && (nd == h.group - 1 || last);
  const bool defer = h.pair && !fuse && !last;
  const size_t set = (size_t)nd * h.L;   // defer: this microbatch's buffers are kdy[set + l], ...
  // cur: gradient entering the layer (never written); its dx goes to the other scratch buffer
  char* top = defer ? pl.kdy[set + h.L - 1] : pl.gA;
  const char* cur = h.head ? top : (const char*)dy;
  char* bufs[2] = {pl.gB, pl.gA};
  int bi = 0;
  if (h.head) {
    char* final_y = h.recompute ? pl.hstash[k] : pl.hacts[mb].y;
    HeadActs& HA = h.recompute ? pl.hacts[0] : pl.hacts[mb];
    if (h.recompute && !head_forward(s, final_y, HA, pl.targets[mb], pl.lossdump)) return STAGE_ERR_DEVICE;
    if (!head_backward(s, final_y, HA, pl.targets[mb], loss_scale, top)) return STAGE_ERR_DEVICE;
  } else if (defer) {   // the caller's dy may be gone by the time the deferred products run
    if (!run(s, "copy", 0, 2.0 * TH, [&] { return copy_bytes(s->st, top, dy, TH); })) return STAGE_ERR_DEVICE;
    cur = top;
  }
  for (int l = h.L - 1; l >= 0; --l) {
    LayerActs& A = h.recompute ? pl.acts[0] : pl.acts[(size_t)mb * h.L + l];
    if (h.recompute && !layer_forward(s, l, in_of(l), A, nullptr)) return STAGE_ERR_DEVICE;
    char* dst = (l == 0 && !h.embed) ? (char*)dx_out : (defer && l > 0) ? pl.kdy[set + l - 1] : bufs[bi];
    WgradPlan wg;
    if (defer) wg.mode = 1;
    if (fuse) {
      wg.mode = 2; wg.nx = nd;
      for (int i = 0; i < nd; ++i) {
        wg.Ax[i] = &pl.acts[(size_t)s->deferred[i] * h.L + l];
        wg.dy_x[i] = pl.kdy[(size_t)i * h.L + l]; wg.dx2_x[i] = pl.kdx2[(size_t)i * h.L + l]; wg.dqkv_x[i] = pl.kdqkv[(size_t)i * h.L + l];
      }
    }
    if (!layer_backward(s, l, in_of(l), A, cur, defer ? pl.kdx2[set + l] : pl.ytmp, dst, defer ? pl.kdqkv[set + l] : pl.gQKV, wg))
      return STAGE_ERR_DEVICE;
    cur = dst;
    bi ^= 1;
  }
  if (fuse) s->deferred.clear();
  if (defer) s->deferred.push_back(mb);
  if (h.embed) {
    // cur now holds the gradient of the embedding output
    if (!run(s, "embed", 0, 3.0 * TH, [&] {
          return embed_bwd(s->st, dt_of(s), h.T, h.H, h.V, pl.ids[mb], cur, s->G(s->seg_off("embed.E"))); }))
      return STAGE_ERR_DEVICE;
  }
  if (h.offload && !mark_computed(s, k)) return STAGE_ERR_DEVICE;
  s->slot[mb] = 2;
  s->pending = mb;
  return STAGE_OK;
}

int stage_accumulate(stage_t* s, int32_t mb) {
  if (!s) return STAGE_ERR_ARG;
  if (!check_slot(s, mb)) return fail(s, STAGE_ERR_ARG, "microbatch slot out of range");
  if (s->pending != mb) return fail(s, STAGE_ERR_STATE, "stage_accumulate must follow stage_backward of the same slot");
  if (!run(s, "reduce_partials", 0, 4.0 * s->plan.partial_floats, [&] {
        return reduce_partials(s->st, s->plan.jobs, s->njobs, s->max_job_width); }))
    return STAGE_ERR_DEVICE;
  s->slot[mb] = 0;
  s->pending = -1;
  s->outstanding--;
  s->accumulated++;
  return STAGE_OK;
}

int stage_graph_replayed(stage_t* s, int32_t n_microbatches) {
  if (!s) return STAGE_ERR_ARG;
  if (n_microbatches < 1 || n_microbatches > s->sh.M) return fail(s, STAGE_ERR_ARG, "n_microbatches must be in 1..max_microbatches");
  if (s->sh.offload) return fail(s, STAGE_ERR_ARG, "calls of a stage with offload_acts = 1 cannot be captured");
  if (s->pending >= 0 || s->outstanding != 0)
    return fail(s, STAGE_ERR_STATE, "microbatches are still outstanding (forward without backward+accumulate)");
  s->accumulated += n_microbatches;
  return STAGE_OK;
}

int stage_optimizer_step(stage_t* s, int64_t t, float grad_scale) {
  if (!s) return STAGE_ERR_ARG;
  if (t < 1) return fail(s, STAGE_ERR_ARG, "t is 1-based");
  if (s->pending >= 0 || s->outstanding != 0)
    return fail(s, STAGE_ERR_STATE, "microbatches are still outstanding (forward without backward+accumulate)");
  if (s->accumulated == 0) return fail(s, STAGE_ERR_STATE, "no microbatch was accumulated since the last step");
  if (!flush_deferred(s)) return STAGE_ERR_DEVICE;
  const stage_config& c = s->cfg;
  AdamW h;
  h.lr = c.lr; h.beta1 = c.beta1; h.beta2 = c.beta2; h.eps = c.adam_eps; h.wd = c.weight_decay;
  h.inv_bc1 = (float)(1.0 / (1.0 - std::pow((double)c.beta1, (double)t)));
  h.inv_bc2 = (float)(1.0 / (1.0 - std::pow((double)c.beta2, (double)t)));
  h.grad_scale = grad_scale;
  h.skip = s->overflow;
  h.zero_grad = false;   // the whole accumulator is cleared by the fill below
  const int64_t P = count_params(c), b = c.shard_begin, e = c.shard_end, n = e - b;
  // loss-scaled training: a non-finite gradient anywhere in the shard raises the flag, and the update that reads
  // the flag then leaves parameters and moments alone
  if (s->overflow && n > 0 && !run(s, "overflow_check", 0, 4.0 * n, [&] { return nonfinite_check(s->st, s->grad + b, n, s->overflow); }))
    return STAGE_ERR_DEVICE;
  const double per = s->sh.bf ? 30.0 : 28.0;
  if (!run(s, "adamw", 0, per * n, [&] {
        return adamw(s->st, dt_of(s), n, b, s->params, s->master, s->grad, s->m, s->v, h); }))
    return STAGE_ERR_DEVICE;
  // The gradients are dropped after the update (Section 4.1.2), those outside the shard too (their owners are the
  // data-parallel peers): one fill over the whole accumulator, after the update has read its range.
  if (!run(s, "zero_grads", 0, 4.0 * P, [&] { return fill_zero(s->st, s->grad, P); })) return STAGE_ERR_DEVICE;
  s->accumulated = 0;
  return STAGE_OK;
}

int stage_set_overflow_flag(stage_t* s, int32_t* device_flag) {
  if (!s) return STAGE_ERR_ARG;
  if ((uintptr_t)device_flag & 3) return fail(s, STAGE_ERR_ARG, "device_flag must be 4-byte aligned");
  s->overflow = (int*)device_flag;
  return STAGE_OK;
}

int stage_loss_scale_update(float* scale, int32_t* good_steps, int32_t found_inf, float backoff, float growth, int32_t growth_interval) {
  if (!scale || !good_steps || !(*scale > 0.f) || !(backoff > 0.f && backoff < 1.f) || !(growth > 1.f) || growth_interval < 1 ||
      *good_steps < 0)
    return fail(nullptr, STAGE_ERR_ARG, "stage_loss_scale_update: scale > 0, 0 < backoff < 1, growth > 1, growth_interval >= 1 required");
  if (found_inf) {
    *scale *= backoff;
    *good_steps = 0;
  } else if (++*good_steps >= growth_interval) {
    *scale *= growth;
    *good_steps = 0;
  }
  return STAGE_OK;
}

int stage_profile(stage_t* s, int32_t enable) {
  if (!s) return STAGE_ERR_ARG;
  s->prof = enable != 0;
  return STAGE_OK;
}

int stage_profile_read(stage_t* s, stage_kernel_stat* out, int32_t n) {
  if (!s || !out || n < 0) return -STAGE_ERR_ARG;
  if (hipStreamSynchronize(s->st) != hipSuccess) return -STAGE_ERR_DEVICE;
  const int nc = (int)s->cls_names.size() < n ? (int)s->cls_names.size() : n;
  for (int i = 0; i < nc; ++i) {
    std::memset(&out[i], 0, sizeof(out[i]));
    std::strncpy(out[i].name, s->cls_names[i].c_str(), sizeof(out[i].name) - 1);
  }
  for (auto& r : s->recs) {
    if (r.cls >= nc) continue;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return -STAGE_ERR_DEVICE;
    out[r.cls].launches++;
    out[r.cls].ms += ms;
    out[r.cls].flops += r.flops;
    out[r.cls].bytes += r.bytes;
  }
  s->recs.clear();
  s->ev_used = 0;
  return nc;
}

int stage_time_layers(stage_t* s, const void* x_or_ids, void* y_out, const void* dy, void* dx_out, const int32_t* targets,
                      float* loss_out, int32_t reps, double* fwd_ms, double* bwd_ms) {
  if (!s) return STAGE_ERR_ARG;
  if (reps < 1 || reps > 1000 || !fwd_ms || !bwd_ms) return fail(s, STAGE_ERR_ARG, "reps must be in 1..1000 and the outputs not NULL");
  if (s->pending >= 0 || s->outstanding != 0 || s->accumulated != 0)
    return fail(s, STAGE_ERR_STATE, "stage_time_layers needs a stage with nothing outstanding and nothing accumulated");
  hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
  for (auto& e : ev)
    if (hipEventCreate(&e) != hipSuccess) return fail(s, STAGE_ERR_DEVICE, "hipEventCreate failed");
  auto done = [&](int rc) {
    for (auto e : ev) (void)hipEventDestroy(e);
    return rc;
  };
  double f = 0.0, b = 0.0;
  const float scale = 1.0f;
  for (int r = -1; r < reps; ++r) {   // round -1 is the warm-up
    if (hipEventRecord(ev[0], s->st) != hipSuccess) return done(fail(s, STAGE_ERR_DEVICE, "hipEventRecord failed"));
    int rc = stage_forward(s, 0, x_or_ids, y_out, targets, loss_out);
    if (rc != STAGE_OK) return done(rc);
    (void)hipEventRecord(ev[1], s->st);
    rc = stage_backward(s, 0, dy, dx_out, scale);
    if (rc == STAGE_OK) rc = stage_accumulate(s, 0);
    if (rc != STAGE_OK) return done(rc);
    (void)hipEventRecord(ev[2], s->st);
    if (hipEventSynchronize(ev[2]) != hipSuccess) return done(fail(s, STAGE_ERR_DEVICE, "hipEventSynchronize failed"));
    float m0 = 0.f, m1 = 0.f;
    if (hipEventElapsedTime(&m0, ev[0], ev[1]) != hipSuccess || hipEventElapsedTime(&m1, ev[1], ev[2]) != hipSuccess)
      return done(fail(s, STAGE_ERR_DEVICE, "hipEventElapsedTime failed"));
    if (r >= 0) { f += m0; b += m1; }
  }
  // give the stage back as it was found: no accumulated microbatch, gradients zero
  if (!flush_deferred(s)) return done(STAGE_ERR_DEVICE);
  s->accumulated = 0;
  if (fill_zero(s->st, s->grad, count_params(s->cfg)) != hipSuccess || hipStreamSynchronize(s->st) != hipSuccess)
    return done(fail(s, STAGE_ERR_DEVICE, "clearing grad_acc failed"));
  *fwd_ms = f / reps;
  *bwd_ms = b / reps;
  return done(STAGE_OK);
}

int stage_fit_linear(const double* x, const double* y, int32_t n, stage_linear_fit* out) {
  if (!x || !y || !out || n < 2) return fail(nullptr, STAGE_ERR_ARG, "stage_fit_linear needs n >= 2 points");
  double xb = 0.0, yb = 0.0;
  for (int i = 0; i < n; ++i) { xb += x[i]; yb += y[i]; }
  xb /= n; yb /= n;
  double sxx = 0.0, sxy = 0.0, syy = 0.0;
  for (int i = 0; i < n; ++i) { sxx += (x[i] - xb) * (x[i] - xb); sxy += (x[i] - xb) * (y[i] - yb); syy += (y[i] - yb) * (y[i] - yb); }
  if (!(sxx > 0.0)) return fail(nullptr, STAGE_ERR_ARG, "stage_fit_linear needs at least two distinct x");
  out->slope = sxy / sxx;
  out->intercept = yb - out->slope * xb;
  double res = 0.0;
  for (int i = 0; i < n; ++i) { const double d = y[i] - (out->intercept + out->slope * x[i]); res += d * d; }
  out->r2 = syy > 0.0 ? 1.0 - res / syy : 1.0;
  return STAGE_OK;
}

const char* stage_last_error(const stage_t* s) { return s ? s->err.c_str() : g_err.c_str(); }

void stage_destroy(stage_t* s) {
  if (!s) return;
  if (s->copy_st) (void)hipStreamSynchronize(s->copy_st);   // no copy may outlive the caller's buffers
  for (auto& d : s->dslot) {
    if (d.copy_done) (void)hipEventDestroy(d.copy_done);
    if (d.compute_done) (void)hipEventDestroy(d.compute_done);
  }
  if (s->copy_st) (void)hipStreamDestroy(s->copy_st);
  for (auto e : s->ev_pool) (void)hipEventDestroy(e);
  delete s;
}

}  // extern "C"
