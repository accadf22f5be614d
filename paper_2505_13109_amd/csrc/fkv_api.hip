// Host side of the C ABI: argument checks, arena carving, per-layer state and the
// stream-ordered schedule of one decode step.  No kernel code here; the one device-side object
// is the library-owned scratch array of the entry point that must not allocate.
#include "../../include/freekv.h"
#include "../../include/freekv_instrument.h"
#include "fkv_internal.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

using namespace fkv;

namespace {

std::string g_create_error;

// Scratch of fkv_sparse_decode_attn_static (split partials, their (m, l) pairs, last-block counters):
// one copy per GPU, held until the process ends.  In host code the array's name is only a handle;
// its device address is looked up once per device (fkv_create) and kept in g_scratch_ptr.
constexpr size_t kStaticScratchBytes = FKV_STATIC_SCRATCH_BYTES;   // 2 MiB
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void* g_scratch_ptr[kMaxDevices] = {};

struct LayerState {
  int L = 0;                 // tokens cached
  int parity = 0;            // which half of the ping-pong buffers is PENDING / staged
  bool have_prev_q = false;  // q_prev valid
  bool have_active = false;  // an ACTIVE selection exists
  bool have_pending = false; // select has run since the last commit
  bool staged_q = false;     // corr_check has run since the last commit
  bool have_flags = false;
  bool offload_outstanding = false;
  bool offload_unseen = false;     // an offload the compute stream has not been made to wait for yet
  bool recall_outstanding = false;
  bool recall_unsubmitted = false; // its deferred recall is still in the context's list, not on the copy stream yet
  hipEvent_t recall_event = nullptr;   // what "that recall finished" is recorded in (its own ev_recall, or a later layer's)
  int recalled = 0;          // placement HOST: which heads' pending pages have been recalled (bit 0 corrected, bit 1 the others)
  int epoch = 0;             // decode steps taken through the one-launch path (selection epochs)
  int last_launches = 0;     // kernel launches of the last fkv_decode_step (compute stream)
  int step_launches = 0;     // launches the last run_step made
  int last_grid = 0;         // grid and dynamic LDS of the last one-launch layer-step
  size_t last_lds = 0;
  hipEvent_t ev_offload = nullptr;   // last page offload finished
  hipEvent_t ev_recall = nullptr;    // deferred recall into ACTIVE's slots finished
};

size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

struct Layout {
  // per layer
  size_t pool, summ, qprev, ids, slots, flags, miss, cosine, counters, tagged, layer_bytes;
  // per context
  size_t P, score, part_o, part_ml, dbg_page, tstamp, bmax, hmax, zsum, cand_key, cand_id, wide_cnt, ctx_bytes;
  size_t total;
  size_t host_layer_bytes, host_total;
  int units_per_head, ring_base, n_ring, sel_base, max_splits, k, max_pages;
};

Layout make_layout(const fkv_config& c) {
  Layout l{};
  const int n_kv = c.n_kv_heads, n_q = c.n_q_heads, b = c.batch;
  l.max_pages = c.max_ctx / PG;
  l.k = (c.budget_tokens - c.sink_tokens - c.window_tokens) / PG;
  l.ring_base = c.sink_tokens / PG;
  l.n_ring = c.window_tokens / PG + 2;
  l.sel_base = l.ring_base + l.n_ring;
  l.units_per_head = c.placement == FKV_PLACE_HBM ? l.max_pages : l.sel_base + 2 * l.k;
  l.max_splits = c.sink_tokens / PG + l.k + c.window_tokens / PG + 1;
  size_t o = 0;
  l.pool = o;   o += align_up((size_t)b * n_kv * l.units_per_head * UNIT_BYTES);
  l.summ = o;   o += align_up((size_t)b * n_kv * 2 * l.max_pages * D * 2);
  l.qprev = o;  o += align_up((size_t)2 * b * n_q * D * 2);
  l.ids = o;    o += align_up((size_t)2 * b * n_kv * (l.k > 0 ? l.k : 1) * 4);
  l.slots = o;  o += align_up((size_t)2 * b * n_kv * (l.k > 0 ? l.k : 1) * 4);
  l.flags = o;  o += align_up((size_t)b * n_kv);
  l.miss = o;   o += align_up((size_t)b * n_kv * (1 + 3 * l.k) * 4);   // per head: count, page ids, slots, positions in the picked list
  l.cosine = o; o += align_up((size_t)b * n_q * 8);
  l.counters = o; o += align_up((size_t)(2 * b * n_kv + 1) * 4);   // last-block counters (selection, attention), then the status word
  l.tagged = o; o += align_up((size_t)b * n_kv * (l.k > 0 ? l.k : 1) * 8);   // epoch-tagged copies of the picked ids (one-launch layer-step)
  l.layer_bytes = o;
  size_t p = 0;
  l.P = p;       p += align_up((size_t)b * n_q * l.max_pages * 4);
  l.score = p;   p += align_up((size_t)b * n_kv * l.max_pages * 4);
  l.part_o = p;  p += align_up((size_t)b * n_kv * l.max_splits * (n_q / n_kv) * D * 4);
  l.part_ml = p; p += align_up((size_t)b * n_kv * l.max_splits * (n_q / n_kv) * 2 * 4);
  l.dbg_page = p; p += align_up((size_t)UNIT_BYTES);
  l.tstamp = p;  p += align_up((size_t)64 * 8);
  // a selection spread over several blocks per head: per-head maxima and integer softmax sums, the slices' short lists
  l.bmax = p;     p += align_up((size_t)b * n_kv * (l.max_pages / 32 + 1) * MAX_G * 4);   // one entry per scoring block of a head
  l.hmax = p;     p += align_up((size_t)b * n_kv * MAX_G * 4);
  l.zsum = p;     p += align_up((size_t)b * n_kv * MAX_G * 8);
  l.cand_key = p; p += align_up((size_t)b * n_kv * WIDE_MAX_SLICES * (l.k > 0 ? l.k : 1) * 4);
  l.cand_id = p;  p += align_up((size_t)b * n_kv * WIDE_MAX_SLICES * (l.k > 0 ? l.k : 1) * 4);
  l.wide_cnt = p; p += align_up((size_t)b * n_kv * 4);
  l.ctx_bytes = p;
  l.total = l.layer_bytes * c.n_layers + l.ctx_bytes;
  l.host_layer_bytes = c.placement == FKV_PLACE_HOST ? (size_t)b * n_kv * l.max_pages * UNIT_BYTES : 0;
  l.host_total = l.host_layer_bytes * c.n_layers;
  return l;
}

const char* check_config(const fkv_config* c) {
  if (!c) return "null config";
  if (c->n_layers < 1 || c->batch < 1) return "n_layers and batch must be >= 1";
  if (c->head_dim != D) return "head_dim must be 128";
  if (c->page_size != PG) return "page_size must be 32";
  if (c->n_kv_heads < 1 || c->n_q_heads < c->n_kv_heads || c->n_q_heads % c->n_kv_heads) return "n_q_heads must be a multiple of n_kv_heads";
  if (c->n_q_heads / c->n_kv_heads > MAX_G) return "group size above 8 is not supported";
  if (c->max_ctx < PG || c->max_ctx % PG) return "max_ctx must be a positive multiple of page_size";
  if (c->budget_tokens % PG || c->sink_tokens % PG || c->window_tokens % PG) return "budget, sink and window must be multiples of page_size";
  if (c->sink_tokens < 0 || c->window_tokens < 0 || c->budget_tokens < c->sink_tokens + c->window_tokens) return "budget must cover sink + window";
  if (c->dtype != FKV_DTYPE_FP16 && c->dtype != FKV_DTYPE_BF16) return "dtype must be fp16 or bf16";
  if (c->placement != FKV_PLACE_HBM && c->placement != FKV_PLACE_HOST) return "bad placement";
  if ((size_t)(c->max_ctx / PG) * 4 + 4096 > 65536) return "max_ctx above 491520 tokens is not supported (top-k keys live in LDS)";
  if ((c->budget_tokens - c->sink_tokens - c->window_tokens) / PG > 1024) return "more than 1024 selectable pages are not supported";
  if (c->placement == FKV_PLACE_HOST && (long)c->batch * c->n_kv_heads > 16384) return "more than 16384 (request, KV head) pairs are not supported with the host pool";
  if (c->tau != c->tau) return "tau is NaN";
  if (c->recall_mode != FKV_RECALL_GATHER && c->recall_mode != FKV_RECALL_MEMCPY) return "bad recall_mode";
  if (c->select_pooling < FKV_POOL_MEAN_S || c->select_pooling > FKV_POOL_MAX_Q) return "bad select_pooling";
  if (c->corr_pooling < FKV_CORR_MEAN || c->corr_pooling > FKV_CORR_MIN) return "bad corr_pooling";
  return nullptr;
}

Geom make_geom(const fkv_config& c, int L) {
  Geom g;
  g.L = L;
  g.n_full = L / PG;
  g.r = L % PG;
  g.n_sink = c.sink_tokens / PG < g.n_full ? c.sink_tokens / PG : g.n_full;
  const int rest = g.n_full - g.n_sink;
  g.n_win = c.window_tokens / PG < rest ? c.window_tokens / PG : rest;
  g.cand_lo = g.n_sink;
  g.n_cand = g.n_full - g.n_sink - g.n_win;
  const int k = (c.budget_tokens - c.sink_tokens - c.window_tokens) / PG;
  g.k_eff = k < g.n_cand ? k : g.n_cand;
  return g;
}

}  // namespace

struct fkv_ctx {
  fkv_config cfg;
  Layout lay;
  Dims dims;
  char* dev = nullptr;
  char* host = nullptr;
  std::vector<LayerState> layers;
  std::string err;
  int device = 0;                     // the HIP device the context was created on
  hipEvent_t ev_fork = nullptr;
  // Deferred recalls of one-launch layer-steps that are not submitted yet: a cross-stream dependency costs the host
  // three HIP calls and each stream a few microseconds, so several layers of a decode step share one.
  std::vector<int> deferred;
  int defer_group = 1;                // layers per submission: a quarter of the layers, so that a recall submitted with the
                                      // group's last layer still has three quarters of a decode step before it is needed;
                                      // at most GATHER_MAX_LAYERS (4, 8 and 16 measure the same on a 32-layer stack)
  hipStream_t deferred_st = nullptr, deferred_cs = nullptr;
  std::vector<std::pair<hipEvent_t, hipStream_t>> waited;   // (recall event, stream that already waits for its latest record)
  uint16_t* nhd_pool = nullptr;       // fkv_attach_nhd_pool: recalled pages also land, converted, in this NHD pool
  int32_t* nhd_slot_pages = nullptr;
  int nhd_slots = 0;
  std::vector<int32_t> host_miss;     // FKV_RECALL_MEMCPY: host copies of the miss lists and flags
  std::vector<uint8_t> host_flags;
  // optional timers around the split attention kernel (fkv_profile_*)
  bool prof_on = false;
  std::vector<hipEvent_t> prof_ev;   // begin/end pairs
  size_t prof_used = 0;

  char* layer_base(int l) const { return dev + lay.layer_bytes * l; }
  char* ctx_base() const { return dev + lay.layer_bytes * cfg.n_layers; }
  PoolDesc pool_desc(int l) const {
    PoolDesc pd;
    pd.pool = reinterpret_cast<uint16_t*>(layer_base(l) + lay.pool);
    pd.units_per_head = lay.units_per_head;
    pd.placement = cfg.placement;
    pd.ring_base = lay.ring_base;
    pd.n_ring = lay.n_ring;
    pd.sel_base = lay.sel_base;
    return pd;
  }
  uint16_t* summ(int l) const { return reinterpret_cast<uint16_t*>(layer_base(l) + lay.summ); }
  uint16_t* host_pool(int l) const { return host ? reinterpret_cast<uint16_t*>(host + lay.host_layer_bytes * l) : nullptr; }
  uint16_t* qprev(int l, int half) const { return reinterpret_cast<uint16_t*>(layer_base(l) + lay.qprev) + (size_t)half * cfg.batch * cfg.n_q_heads * D; }
  int32_t* ids(int l, int half) const { return reinterpret_cast<int32_t*>(layer_base(l) + lay.ids) + (size_t)half * cfg.batch * cfg.n_kv_heads * (lay.k > 0 ? lay.k : 1); }
  int32_t* slots(int l, int half) const { return reinterpret_cast<int32_t*>(layer_base(l) + lay.slots) + (size_t)half * cfg.batch * cfg.n_kv_heads * (lay.k > 0 ? lay.k : 1); }
  uint8_t* flags(int l) const { return reinterpret_cast<uint8_t*>(layer_base(l) + lay.flags); }
  int32_t* miss(int l) const { return reinterpret_cast<int32_t*>(layer_base(l) + lay.miss); }
  double* cosine(int l) const { return reinterpret_cast<double*>(layer_base(l) + lay.cosine); }
  int* sel_counters(int l) const { return reinterpret_cast<int*>(layer_base(l) + lay.counters); }
  int* attn_counters(int l) const { return reinterpret_cast<int*>(layer_base(l) + lay.counters) + cfg.batch * cfg.n_kv_heads; }
  unsigned long long* tagged(int l) const { return reinterpret_cast<unsigned long long*>(layer_base(l) + lay.tagged); }
  int* status(int l) const { return reinterpret_cast<int*>(layer_base(l) + lay.counters) + 2 * cfg.batch * cfg.n_kv_heads; }
  float* P() const { return reinterpret_cast<float*>(ctx_base() + lay.P); }
  float* score() const { return reinterpret_cast<float*>(ctx_base() + lay.score); }
  float* part_o() const { return reinterpret_cast<float*>(ctx_base() + lay.part_o); }
  float* part_ml() const { return reinterpret_cast<float*>(ctx_base() + lay.part_ml); }
  uint16_t* dbg_page() const { return reinterpret_cast<uint16_t*>(ctx_base() + lay.dbg_page); }
  bool lose_selection = false;   // fkv_test_lose_selection: corrected heads' attention waits in vain (tests the bounded wait)
  bool stamp_on = false;   // fkv_instrument_timestamps: kernels record phase timestamps of head 0 (debugging aid)
  long long* tstamp() const { return stamp_on ? reinterpret_cast<long long*>(ctx_base() + lay.tstamp) : nullptr; }

  int fail(int code, const std::string& msg) { err = msg; return code; }
  int hip_fail(hipError_t e, const char* what) {
    err = std::string(what) + ": " + hipGetErrorString(e);
    return FKV_EHIP;
  }
};

#define FKV_HIP(ctx, call)                                   \
  do {                                                       \
    hipError_t e_ = (call);                                  \
    if (e_ != hipSuccess) return (ctx)->hip_fail(e_, #call); \
  } while (0)

#define FKV_CHECK_LAYER(ctx, layer)                                                  \
  do {                                                                               \
    if (!(ctx)) return FKV_EINVAL;                                                   \
    if ((layer) < 0 || (layer) >= (ctx)->cfg.n_layers) return (ctx)->fail(FKV_ERANGE, "layer out of range"); \
  } while (0)

// Work of this layer on `st` from here on must see the deferred recall of the previous
// step finished: it reuses the miss list and flags that recall reads, and the slots it fills.
static int wait_recall(fkv_ctx* ctx, LayerState& ls, hipStream_t st) {
  if (ls.recall_outstanding) {
    // Layers whose recalls were submitted together share the event: the stream waits for it once, with the first of
    // them that comes round again (a dependency between streams costs the host and the waiting stream microseconds
    // even when it is satisfied long since, as it is here: the recall had a whole decode step).
    bool covered = false;
    for (const auto& w : ctx->waited)
      if (w.first == ls.recall_event && w.second == st) covered = true;
    if (!covered) {
      hipError_t e = hipStreamWaitEvent(st, ls.recall_event, 0);
      if (e != hipSuccess) return ctx->hip_fail(e, "hipStreamWaitEvent");
      ctx->waited.emplace_back(ls.recall_event, st);
    }
    ls.recall_outstanding = false;
  }
  return FKV_OK;
}

static const void* ctx_base_tstamp(const fkv_ctx* ctx) { return ctx->ctx_base() + ctx->lay.tstamp; }

static int after_launch(fkv_ctx* ctx, const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return ctx->hip_fail(e, what);
  return FKV_OK;
}

// One launch of the step kernel with the given roles (append / correction test / selection).
static StepIO make_step_io(fkv_ctx* ctx, int layer, const void* q, const void* k_new, const void* v_new,
                           uint8_t* flags_user, int32_t* ids_user) {
  LayerState& ls = ctx->layers[layer];
  StepIO io{};
  io.pd = ctx->pool_desc(layer);
  io.summ = ctx->summ(layer);
  io.k_new = static_cast<const uint16_t*>(k_new);
  io.v_new = static_cast<const uint16_t*>(v_new);
  io.q = static_cast<const uint16_t*>(q);
  io.q_prev = ctx->qprev(layer, ls.parity ^ 1);
  io.q_stage = ctx->qprev(layer, ls.parity);
  io.have_prev = ls.have_prev_q ? 1 : 0;
  io.tau = ctx->cfg.tau;
  io.flags = ctx->flags(layer);
  io.flags_user = flags_user;
  io.cosine = ctx->cosine(layer);
  io.P = ctx->P();
  io.score = ctx->score();
  io.ids = ctx->ids(layer, ls.parity);
  io.ids_user = ids_user;
  io.counters = ctx->sel_counters(layer);
  io.tstamp = ctx->tstamp();
  char* cb = ctx->ctx_base();
  io.bmax = reinterpret_cast<float*>(cb + ctx->lay.bmax);
  io.bmax_stride = ctx->lay.max_pages / 32 + 1;
  io.hmax = reinterpret_cast<float*>(cb + ctx->lay.hmax);
  io.zsum = reinterpret_cast<unsigned long long*>(cb + ctx->lay.zsum);
  io.cand_key = reinterpret_cast<uint32_t*>(cb + ctx->lay.cand_key);
  io.cand_id = reinterpret_cast<int32_t*>(cb + ctx->lay.cand_id);
  io.wide_counters = reinterpret_cast<int*>(cb + ctx->lay.wide_cnt);
  if (ctx->cfg.placement == FKV_PLACE_HOST) {      // a selection comes with its recall plan
    io.plan_act_ids = ctx->ids(layer, ls.parity ^ 1);
    io.plan_act_slots = ctx->slots(layer, ls.parity ^ 1);
    io.plan_new_slots = ctx->slots(layer, ls.parity);
    io.plan_miss = ctx->miss(layer);
  }
  return io;
}

static int run_step(fkv_ctx* ctx, int layer, int roles, const void* q, const void* k_new, const void* v_new,
                    uint8_t* flags_user, int32_t* ids_user, int L_after, hipStream_t st) {
  const StepIO io = make_step_io(ctx, layer, q, k_new, v_new, flags_user, ids_user);
  LayerState& ls = ctx->layers[layer];
  ls.step_launches = launch_step(ctx->dims, roles, io, make_geom(ctx->cfg, L_after), st);
  if ((roles & ROLE_SELECT) && io.plan_new_slots) ls.recalled = 0;     // a new plan: nothing of it is recalled yet
  return after_launch(ctx, "step kernel");
}

// Host-side bookkeeping after an append has been enqueued; placement HOST offloads a page
// the token filled (Sec. 4.2), behind the append, on the copy stream.
static int after_append(fkv_ctx* ctx, int layer, hipStream_t st, hipStream_t cs) {
  LayerState& ls = ctx->layers[layer];
  ls.L += 1;
  if (ctx->cfg.placement == FKV_PLACE_HOST && ls.L % PG == 0) {
    if (cs != st) {
      FKV_HIP(ctx, hipEventRecord(ctx->ev_fork, st));
      FKV_HIP(ctx, hipStreamWaitEvent(cs, ctx->ev_fork, 0));
    }
    launch_offload(ctx->dims, ctx->pool_desc(layer), ctx->host_pool(layer), ls.L / PG - 1, cs);
    int rc = after_launch(ctx, "offload kernel");
    if (rc) return rc;
    FKV_HIP(ctx, hipEventRecord(ls.ev_offload, cs));
    ls.offload_outstanding = true;
    ls.offload_unseen = cs != st;
  }
  return FKV_OK;
}

static int run_plan(fkv_ctx* ctx, int layer, hipStream_t st) {
  LayerState& ls = ctx->layers[layer];
  if (ctx->cfg.placement != FKV_PLACE_HOST) return FKV_OK;
  launch_plan(ctx->dims, ctx->ids(layer, ls.parity), ctx->ids(layer, ls.parity ^ 1), ctx->slots(layer, ls.parity ^ 1),
              ctx->slots(layer, ls.parity), ctx->miss(layer), ls.L / PG, st);
  ls.recalled = 0;
  return after_launch(ctx, "plan kernel");
}

static void forget_waits(fkv_ctx* ctx, hipEvent_t ev) {     // `ev` has just been recorded again
  auto& w = ctx->waited;
  for (size_t i = 0; i < w.size();)
    if (w[i].first == ev) { w[i] = w.back(); w.pop_back(); } else ++i;
}

// Submit the deferred recalls on the list: one dependency of the copy stream on the compute stream, one gather launch
// for all listed layers' uncorrected heads, one event that every listed layer's next step looks at.
static int flush_deferred(fkv_ctx* ctx) {
  if (ctx->deferred.empty()) return FKV_OK;
  hipStream_t st = ctx->deferred_st, cs = ctx->deferred_cs;
  if (cs != st) {
    FKV_HIP(ctx, hipEventRecord(ctx->ev_fork, st));
    FKV_HIP(ctx, hipStreamWaitEvent(cs, ctx->ev_fork, 0));
  }
  for (size_t i0 = 0; i0 < ctx->deferred.size(); i0 += GATHER_MAX_LAYERS) {
    GatherLayers gl{};
    for (size_t i = i0; i < ctx->deferred.size() && gl.n < GATHER_MAX_LAYERS; ++i) {
      const int l = ctx->deferred[i];
      gl.pd[gl.n] = ctx->pool_desc(l);
      gl.host_pool[gl.n] = ctx->host_pool(l);
      gl.miss[gl.n] = ctx->miss(l);
      gl.flags[gl.n] = ctx->flags(l);
      gl.n += 1;
    }
    launch_gather(ctx->dims, gl, FKV_HEADS_UNFLAGGED, cs);
  }
  int rc = after_launch(ctx, "gather kernel");
  if (rc) return rc;
  hipEvent_t done = ctx->layers[ctx->deferred.back()].ev_recall;
  if (cs != st) {
    FKV_HIP(ctx, hipEventRecord(done, cs));
    forget_waits(ctx, done);
  }
  for (int l : ctx->deferred) {
    LayerState& ls = ctx->layers[l];
    ls.recall_unsubmitted = false;
    ls.recall_event = done;
    ls.recall_outstanding = cs != st;
  }
  ctx->deferred.clear();
  return FKV_OK;
}
// every entry point that looks at or changes a layer's state first submits what is on the list
#define FKV_FLUSH(ctx)                          \
  do {                                          \
    if ((ctx) && !(ctx)->deferred.empty()) {    \
      int rc_ = flush_deferred(ctx);            \
      if (rc_) return rc_;                      \
    }                                           \
  } while (0)

extern "C" {

int fkv_arena_bytes(const fkv_config* cfg, size_t* dev_bytes, size_t* host_bytes) {
  const char* why = check_config(cfg);
  if (why) { g_create_error = why; return FKV_EINVAL; }
  const Layout l = make_layout(*cfg);
  if (dev_bytes) *dev_bytes = l.total;
  if (host_bytes) *host_bytes = l.host_total;
  return FKV_OK;
}

int fkv_create(const fkv_config* cfg, void* dev_arena, size_t dev_bytes, void* host_arena,
               size_t host_bytes, fkv_ctx** out) {
  if (!out) { g_create_error = "null out pointer"; return FKV_EINVAL; }
  *out = nullptr;
  const char* why = check_config(cfg);
  if (why) { g_create_error = why; return FKV_EINVAL; }
  const Layout l = make_layout(*cfg);
  if (!dev_arena || (reinterpret_cast<uintptr_t>(dev_arena) & 255)) { g_create_error = "device arena null or not 256-byte aligned"; return FKV_EINVAL; }
  if (dev_bytes < l.total) { g_create_error = "device arena too small"; return FKV_ENOMEM; }
  if (cfg->placement == FKV_PLACE_HOST) {
    if (!host_arena || (reinterpret_cast<uintptr_t>(host_arena) & 255)) { g_create_error = "host arena null or not 256-byte aligned"; return FKV_EINVAL; }
    if (host_bytes < l.host_total) { g_create_error = "host arena too small"; return FKV_ENOMEM; }
  }
  fkv_ctx* ctx = new fkv_ctx();
  ctx->cfg = *cfg;
  ctx->lay = l;
  int dev_id = 0, max_lds = 65536;
  if (hipGetDevice(&dev_id) != hipSuccess || dev_id < 0 || dev_id >= kMaxDevices) {
    g_create_error = "no current HIP device";
    delete ctx;
    return FKV_EHIP;
  }
  ctx->device = dev_id;
  if (!g_scratch_ptr[dev_id]) {     // this device's copy of the static scratch array
    void* ptr = nullptr;
    const hipError_t es = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (es != hipSuccess || !ptr) {
      g_create_error = std::string("hipGetSymbolAddress(scratch): ") + hipGetErrorString(es);
      delete ctx;
      return FKV_EHIP;
    }
    g_scratch_ptr[dev_id] = ptr;
  }
  {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev_id) == hipSuccess && v > 0) max_lds = v;
    v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeSharedMemPerBlockOptin, dev_id) == hipSuccess && v > max_lds) max_lds = v;
  }
  ctx->dims = Dims{cfg->batch, cfg->n_q_heads, cfg->n_kv_heads, cfg->n_q_heads / cfg->n_kv_heads, l.k, l.max_pages, cfg->dtype, max_lds,
                   cfg->select_pooling, cfg->corr_pooling};
  ctx->dev = static_cast<char*>(dev_arena);
  ctx->host = cfg->placement == FKV_PLACE_HOST ? static_cast<char*>(host_arena) : nullptr;
  ctx->layers.resize(cfg->n_layers);
  ctx->defer_group = cfg->n_layers / 4 < 1 ? 1 : cfg->n_layers / 4 > GATHER_MAX_LAYERS ? GATHER_MAX_LAYERS : cfg->n_layers / 4;
  hipError_t e = hipMemset(dev_arena, 0, l.total);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  const unsigned ev_flags = hipEventDisableTiming;
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_fork, ev_flags);
  for (int i = 0; e == hipSuccess && i < cfg->n_layers; ++i) {
    e = hipEventCreateWithFlags(&ctx->layers[i].ev_offload, ev_flags);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->layers[i].ev_recall, ev_flags);
  }
  if (e != hipSuccess) {
    g_create_error = std::string("HIP failure in fkv_create: ") + hipGetErrorString(e);
    fkv_destroy(ctx);
    return FKV_EHIP;
  }
  // ids start as "nothing picked"
  for (int i = 0; i < cfg->n_layers; ++i) {
    const size_t n = (size_t)2 * cfg->batch * cfg->n_kv_heads * (l.k > 0 ? l.k : 1) * 4;
    e = hipMemset(ctx->ids(i, 0), 0xff, n);
    if (e != hipSuccess) break;
  }
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    g_create_error = std::string("HIP failure in fkv_create: ") + hipGetErrorString(e);
    fkv_destroy(ctx);
    return FKV_EHIP;
  }
  *out = ctx;
  return FKV_OK;
}

int fkv_destroy(fkv_ctx* ctx) {
  if (!ctx) return FKV_EINVAL;
  (void)hipDeviceSynchronize();
  if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
  for (hipEvent_t e : ctx->prof_ev) (void)hipEventDestroy(e);
  for (auto& ls : ctx->layers) {
    if (ls.ev_offload) (void)hipEventDestroy(ls.ev_offload);
    if (ls.ev_recall) (void)hipEventDestroy(ls.ev_recall);
  }
  delete ctx;
  return FKV_OK;
}

const char* fkv_last_error(const fkv_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

int fkv_step_launches(const fkv_ctx* ctx, int32_t layer) {
  if (!ctx) return FKV_EINVAL;
  if (layer < 0 || layer >= ctx->cfg.n_layers) return FKV_ERANGE;
  return ctx->layers[layer].last_launches;
}

int fkv_context_len(const fkv_ctx* ctx, int32_t layer) {
  if (!ctx) return FKV_EINVAL;
  if (layer < 0 || layer >= ctx->cfg.n_layers) return FKV_ERANGE;
  return ctx->layers[layer].L;
}

int fkv_health(fkv_ctx* ctx, int32_t layer) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  int flag = 0;
  FKV_HIP(ctx, hipDeviceSynchronize());
  FKV_HIP(ctx, hipMemcpy(&flag, ctx->status(layer), sizeof(int), hipMemcpyDeviceToHost));
  if (flag != 0) {
    FKV_HIP(ctx, hipMemset(ctx->status(layer), 0, sizeof(int)));
    return ctx->fail(FKV_ETIMEOUT, "an attention block gave up waiting for its head's selection");
  }
  return FKV_OK;
}

int fkv_load_prefix(fkv_ctx* ctx, int32_t layer, const void* K_dev, const void* V_dev, int32_t n_tokens, void* stream) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  if (n_tokens < 0 || n_tokens > ctx->cfg.max_ctx) return ctx->fail(FKV_ERANGE, "n_tokens exceeds max_ctx");
  if (n_tokens > 0 && (!K_dev || !V_dev)) return ctx->fail(FKV_EINVAL, "null K or V");
  LayerState& ls = ctx->layers[layer];
  hipStream_t st = static_cast<hipStream_t>(stream);
  const Geom g = make_geom(ctx->cfg, n_tokens);
  launch_load_prefix(ctx->dims, ctx->pool_desc(layer), ctx->summ(layer), ctx->host_pool(layer),
                     static_cast<const uint16_t*>(K_dev), static_cast<const uint16_t*>(V_dev), n_tokens, g, st);
  int rc = after_launch(ctx, "load_prefix kernel");
  if (rc) return rc;
  // a fresh context: no previous query, nothing picked
  const size_t n = (size_t)2 * ctx->cfg.batch * ctx->cfg.n_kv_heads * (ctx->lay.k > 0 ? ctx->lay.k : 1) * 4;
  FKV_HIP(ctx, hipMemsetAsync(ctx->ids(layer, 0), 0xff, n, st));
  ls.L = n_tokens;
  ls.parity = 0;
  ls.have_prev_q = ls.have_active = ls.have_pending = ls.staged_q = ls.have_flags = false;
  ls.offload_outstanding = ls.recall_outstanding = false;
  ls.recalled = 0;
  return FKV_OK;
}

int fkv_kv_append(fkv_ctx* ctx, int32_t layer, const void* k_new_dev, const void* v_new_dev, void* stream, void* copy_stream) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  if (!k_new_dev || !v_new_dev) return ctx->fail(FKV_EINVAL, "null k_new or v_new");
  LayerState& ls = ctx->layers[layer];
  if (ls.L >= ctx->cfg.max_ctx) return ctx->fail(FKV_ERANGE, "append beyond max_ctx");
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = run_step(ctx, layer, ROLE_APPEND, nullptr, k_new_dev, v_new_dev, nullptr, nullptr, ls.L + 1, st);
  if (rc) return rc;
  return after_append(ctx, layer, st, static_cast<hipStream_t>(copy_stream));
}

int fkv_page_summary_update(fkv_ctx* ctx, int32_t layer, int32_t first_page, int32_t n_pages, void* stream) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  if (ctx->cfg.placement != FKV_PLACE_HBM) return ctx->fail(FKV_ESTATE, "summary recompute needs the keys in HBM");
  LayerState& ls = ctx->layers[layer];
  const int n_have = (ls.L + PG - 1) / PG;
  if (first_page < 0 || n_pages < 0 || first_page + n_pages > n_have) return ctx->fail(FKV_ERANGE, "page range beyond the cached context");
  launch_summary_recompute(ctx->dims, ctx->pool_desc(layer), ctx->summ(layer), first_page, n_pages,
                           make_geom(ctx->cfg, ls.L), static_cast<hipStream_t>(stream));
  return after_launch(ctx, "summary kernel");
}

int fkv_corr_check(fkv_ctx* ctx, int32_t layer, const void* q_dev, uint8_t* flags_dev, void* stream) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  if (!q_dev) return ctx->fail(FKV_EINVAL, "null q");
  LayerState& ls = ctx->layers[layer];
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = wait_recall(ctx, ls, st);
  if (rc) return rc;
  rc = run_step(ctx, layer, ROLE_CORR, q_dev, nullptr, nullptr, flags_dev, nullptr, ls.L, st);
  if (rc) return rc;
  ls.staged_q = true;
  ls.have_flags = true;
  return FKV_OK;
}

int fkv_page_select(fkv_ctx* ctx, int32_t layer, const void* q_dev, int32_t* page_ids_dev, void* stream) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  if (!q_dev) return ctx->fail(FKV_EINVAL, "null q");
  LayerState& ls = ctx->layers[layer];
  if (ls.L < 1) return ctx->fail(FKV_ESTATE, "empty context");
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = wait_recall(ctx, ls, st);
  if (rc) return rc;
  rc = run_step(ctx, layer, ROLE_SELECT, q_dev, nullptr, nullptr, nullptr, page_ids_dev, ls.L, st);
  if (rc) return rc;
  ls.have_pending = true;
  return FKV_OK;
}

// copy the missing pages of the PENDING selection's chosen heads (by flag or by mask) into their slots
static int recall_missing(fkv_ctx* ctx, int layer, int heads_mode, const uint8_t* select_by, hipStream_t cs) {
  LayerState& ls = ctx->layers[layer];
  if (ls.offload_outstanding) {   // a page offloaded moments ago may be picked already
    FKV_HIP(ctx, hipStreamWaitEvent(cs, ls.ev_offload, 0));
  }
  if (ctx->cfg.recall_mode == FKV_RECALL_MEMCPY) {
    if (ctx->nhd_pool) return ctx->fail(FKV_ESTATE, "the streamed NHD recall needs recall_mode GATHER");
    // the miss lists and flags come to the host (blocking), then one copy per 16 KiB unit
    const fkv_config& c = ctx->cfg;
    const int n_heads = c.batch * c.n_kv_heads, kk = ctx->lay.k;
    const size_t n_int = (size_t)n_heads * (1 + 3 * kk);
    if (ctx->host_miss.size() < n_int) ctx->host_miss.resize(n_int);
    if (ctx->host_flags.size() < (size_t)n_heads) ctx->host_flags.resize(n_heads);
    FKV_HIP(ctx, hipMemcpyAsync(ctx->host_miss.data(), ctx->miss(layer), n_int * 4, hipMemcpyDeviceToHost, cs));
    if (heads_mode != FKV_HEADS_ALL)
      FKV_HIP(ctx, hipMemcpyAsync(ctx->host_flags.data(), select_by, n_heads, hipMemcpyDeviceToHost, cs));
    FKV_HIP(ctx, hipStreamSynchronize(cs));
    const PoolDesc pd = ctx->pool_desc(layer);
    for (int h = 0; h < n_heads; ++h) {
      if (heads_mode != FKV_HEADS_ALL && ((heads_mode == FKV_HEADS_FLAGGED) != (ctx->host_flags[h] != 0))) continue;
      const int32_t* mh = ctx->host_miss.data() + (size_t)h * (1 + 3 * kk);
      for (int i = 0; i < mh[0]; ++i) {
        const uint16_t* src = ctx->host_pool(layer) + ((size_t)h * ctx->lay.max_pages + mh[1 + i]) * UNIT_ELEMS;
        uint16_t* dst = pd.pool + ((size_t)h * pd.units_per_head + pd.sel_base + mh[1 + kk + i]) * UNIT_ELEMS;
        FKV_HIP(ctx, hipMemcpyAsync(dst, src, UNIT_BYTES, hipMemcpyHostToDevice, cs));
      }
    }
    return FKV_OK;
  }
  if (ctx->nhd_pool) {
    // streamed recall: host unit -> LDS staging -> page-cache slot and NHD rows (Sec. 4.2)
    launch_gather_nhd(ctx->dims, ctx->pool_desc(layer), ctx->host_pool(layer), ctx->miss(layer), select_by, heads_mode,
                      ctx->nhd_pool, ctx->nhd_slots, make_geom(ctx->cfg, ls.L).n_sink, cs);
    return after_launch(ctx, "streamed NHD gather kernel");
  }
  GatherLayers gl{};
  gl.n = 1;
  gl.pd[0] = ctx->pool_desc(layer); gl.host_pool[0] = ctx->host_pool(layer); gl.miss[0] = ctx->miss(layer); gl.flags[0] = select_by;
  launch_gather(ctx->dims, gl, heads_mode, cs);
  return after_launch(ctx, "gather kernel");
}

int fkv_recall_pending(fkv_ctx* ctx, int32_t layer, int32_t heads, void* copy_stream) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  if (heads < 0 || heads > 2) return ctx->fail(FKV_EINVAL, "bad heads selector");
  if (ctx->cfg.placement != FKV_PLACE_HOST) return FKV_OK;
  LayerState& ls = ctx->layers[layer];
  if (!ls.have_pending) return ctx->fail(FKV_ESTATE, "recall before page_select");
  if (heads != FKV_HEADS_ALL && !ls.have_flags) return ctx->fail(FKV_ESTATE, "recall by flag before corr_check");
  int rc = recall_missing(ctx, layer, heads, ctx->flags(layer), static_cast<hipStream_t>(copy_stream));
  if (rc) return rc;
  ls.recalled |= heads == FKV_HEADS_ALL ? 3 : heads == FKV_HEADS_FLAGGED ? 1 : 2;
  return FKV_OK;
}

int fkv_recall_pages(fkv_ctx* ctx, int32_t layer, const int32_t* page_ids_dev, const uint8_t* head_mask_dev, void* copy_stream) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  if (ctx->cfg.placement != FKV_PLACE_HOST) return FKV_OK;
  LayerState& ls = ctx->layers[layer];
  hipStream_t cs = static_cast<hipStream_t>(copy_stream);
  if (page_ids_dev) {
    // the caller's list becomes the PENDING selection: planned against ACTIVE's slots like one of the library's own
    if (ls.L < 1) return ctx->fail(FKV_ESTATE, "empty context");
    int rc = wait_recall(ctx, ls, cs);
    if (rc) return rc;
    const size_t n = (size_t)ctx->cfg.batch * ctx->cfg.n_kv_heads * ctx->lay.k * sizeof(int32_t);
    if (n) FKV_HIP(ctx, hipMemcpyAsync(ctx->ids(layer, ls.parity), page_ids_dev, n, hipMemcpyDeviceToDevice, cs));
    rc = run_plan(ctx, layer, cs);
    if (rc) return rc;
    ls.have_pending = true;
  } else if (!ls.have_pending) {
    return ctx->fail(FKV_ESTATE, "recall of the pending selection before page_select");
  }
  int rc = recall_missing(ctx, layer, head_mask_dev ? FKV_HEADS_FLAGGED : FKV_HEADS_ALL, head_mask_dev, cs);
  if (rc) return rc;
  if (!head_mask_dev) ls.recalled = 3;
  return FKV_OK;
}

int fkv_sparse_decode_attn(fkv_ctx* ctx, int32_t layer, const void* q_dev, float* out_dev, int32_t use, void* stream) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  if (!q_dev || !out_dev) return ctx->fail(FKV_EINVAL, "null q or out");
  if (use < 0 || use > 2) return ctx->fail(FKV_EINVAL, "bad use selector");
  LayerState& ls = ctx->layers[layer];
  if (ls.L < 1) return ctx->fail(FKV_ESTATE, "empty context");
  if (use != FKV_USE_ACTIVE && !ls.have_pending) return ctx->fail(FKV_ESTATE, "attention on the pending selection before page_select");
  if (use == FKV_USE_BY_FLAG && !ls.have_flags) return ctx->fail(FKV_ESTATE, "attention by flag before corr_check");
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rcw = wait_recall(ctx, ls, st);
  if (rcw) return rcw;
  const Geom g = make_geom(ctx->cfg, ls.L);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (ctx->prof_on && ctx->prof_used + 2 <= ctx->prof_ev.size()) {
    e0 = ctx->prof_ev[ctx->prof_used++];
    e1 = ctx->prof_ev[ctx->prof_used++];
  }
  launch_attn(ctx->dims, ctx->pool_desc(layer), static_cast<const uint16_t*>(q_dev), ctx->ids(layer, ls.parity ^ 1),
              ctx->ids(layer, ls.parity), ctx->slots(layer, ls.parity ^ 1), ctx->slots(layer, ls.parity),
              ctx->flags(layer), use, ctx->part_o(), ctx->part_ml(), ctx->lay.max_splits, ctx->attn_counters(layer),
              out_dev, g, st, e0, e1, ctx->tstamp());
  return after_launch(ctx, "attention kernels");
}

int fkv_sparse_decode_attn_static(fkv_ctx* ctx, int32_t layer, const void* q_dev, float* out_dev, int32_t use, void* stream) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  if (!q_dev || !out_dev) return ctx->fail(FKV_EINVAL, "null q or out");
  if (use < 0 || use > 2) return ctx->fail(FKV_EINVAL, "bad use selector");
  LayerState& ls = ctx->layers[layer];
  if (ls.L < 1) return ctx->fail(FKV_ESTATE, "empty context");
  if (use != FKV_USE_ACTIVE && !ls.have_pending) return ctx->fail(FKV_ESTATE, "attention on the pending selection before page_select");
  if (use == FKV_USE_BY_FLAG && !ls.have_flags) return ctx->fail(FKV_ESTATE, "attention by flag before corr_check");
  char* base = static_cast<char*>(g_scratch_ptr[ctx->device]);
  if (!base) return ctx->fail(FKV_ESTATE, "no static scratch on this device");
  // the split this shape takes, and what its partials need (stride = the splits actually written)
  const fkv_config& c = ctx->cfg;
  const Geom g = make_geom(c, ls.L);
  const int heads = c.batch * c.n_kv_heads, G = c.n_q_heads / c.n_kv_heads;
  const int n_att = g.n_sink + ctx->lay.k + g.n_win + (g.r > 0 ? 1 : 0);
  const int pps = attn_pages_per_block(n_att, heads, ctx->lay.max_splits, 4);
  const int n_splits = (n_att + pps - 1) / pps;
  const size_t b_cnt = align_up((size_t)heads * sizeof(int));
  const size_t b_ml = align_up((size_t)heads * n_splits * G * 2 * sizeof(float));
  const size_t b_o = align_up((size_t)heads * n_splits * G * D * sizeof(float));
  if (b_cnt + b_ml + b_o > kStaticScratchBytes) {
    char msg[160];
    snprintf(msg, sizeof msg, "static scratch too small: this shape needs %zu bytes, the library holds %zu", b_cnt + b_ml + b_o,
             kStaticScratchBytes);
    return ctx->fail(FKV_ENOMEM, msg);
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rcw = wait_recall(ctx, ls, st);
  if (rcw) return rcw;
  // the array keeps the last call's contents: the counters must start at zero (a fill kernel, not a
  // memset node, so that the call can be captured into a graph)
  launch_fill_zero(reinterpret_cast<int*>(base), heads, st);
  launch_attn(ctx->dims, ctx->pool_desc(layer), static_cast<const uint16_t*>(q_dev), ctx->ids(layer, ls.parity ^ 1),
              ctx->ids(layer, ls.parity), ctx->slots(layer, ls.parity ^ 1), ctx->slots(layer, ls.parity),
              ctx->flags(layer), use, reinterpret_cast<float*>(base + b_cnt + b_ml), reinterpret_cast<float*>(base + b_cnt),
              n_splits, reinterpret_cast<int*>(base), out_dev, g, st, nullptr, nullptr, nullptr);
  return after_launch(ctx, "attention kernels (static scratch)");
}

int fkv_export_nhd(fkv_ctx* ctx, int32_t layer, int32_t use, void* nhd_pool_dev, int32_t* slot_pages_dev,
                   int32_t n_slots, void* stream) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  if (!nhd_pool_dev || !slot_pages_dev) return ctx->fail(FKV_EINVAL, "null output");
  if (use < 0 || use > 2) return ctx->fail(FKV_EINVAL, "bad use selector");
  const fkv_config& c = ctx->cfg;
  if (n_slots != c.budget_tokens / c.page_size + 1) return ctx->fail(FKV_EINVAL, "n_slots must be budget/page + 1");
  if ((reinterpret_cast<uintptr_t>(nhd_pool_dev) & 15) != 0) return ctx->fail(FKV_EINVAL, "pool not 16-byte aligned");
  LayerState& ls = ctx->layers[layer];
  if (ls.L < 1) return ctx->fail(FKV_ESTATE, "empty context");
  if (use == FKV_USE_ACTIVE && ctx->lay.k > 0 && !ls.have_active) return ctx->fail(FKV_ESTATE, "no active selection yet");
  if (use != FKV_USE_ACTIVE && !ls.have_pending) return ctx->fail(FKV_ESTATE, "export of the pending selection before page_select");
  if (use == FKV_USE_BY_FLAG && !ls.have_flags) return ctx->fail(FKV_ESTATE, "export by flag before corr_check");
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rcw = wait_recall(ctx, ls, st);
  if (rcw) return rcw;
  launch_export_nhd(ctx->dims, ctx->pool_desc(layer), ctx->ids(layer, ls.parity ^ 1), ctx->ids(layer, ls.parity),
                    ctx->slots(layer, ls.parity ^ 1), ctx->slots(layer, ls.parity), ctx->flags(layer), use,
                    static_cast<uint16_t*>(nhd_pool_dev), slot_pages_dev, n_slots, make_geom(c, ls.L), st);
  return after_launch(ctx, "NHD export kernel");
}

int fkv_attach_nhd_pool(fkv_ctx* ctx, void* nhd_pool_dev, int32_t* slot_pages_dev, int32_t n_slots) {
  if (!ctx) return FKV_EINVAL;
  FKV_FLUSH(ctx);
  if (!nhd_pool_dev) {
    ctx->nhd_pool = nullptr; ctx->nhd_slot_pages = nullptr; ctx->nhd_slots = 0;
    return FKV_OK;
  }
  const fkv_config& c = ctx->cfg;
  if (c.placement != FKV_PLACE_HOST) return ctx->fail(FKV_ESTATE, "the streamed NHD recall is for the host-pool placement");
  if (c.recall_mode != FKV_RECALL_GATHER) return ctx->fail(FKV_ESTATE, "the streamed NHD recall needs recall_mode GATHER");
  if (!slot_pages_dev) return ctx->fail(FKV_EINVAL, "null slot_pages");
  if (n_slots != c.budget_tokens / c.page_size + 1) return ctx->fail(FKV_EINVAL, "n_slots must be budget/page + 1");
  if ((reinterpret_cast<uintptr_t>(nhd_pool_dev) & 15) != 0) return ctx->fail(FKV_EINVAL, "pool not 16-byte aligned");
  ctx->nhd_pool = static_cast<uint16_t*>(nhd_pool_dev);
  ctx->nhd_slot_pages = slot_pages_dev;
  ctx->nhd_slots = n_slots;
  return FKV_OK;
}

static int commit_layer(fkv_ctx* ctx, int32_t layer) {
  LayerState& ls = ctx->layers[layer];
  if (!ls.have_pending || !ls.staged_q) return ctx->fail(FKV_ESTATE, "commit needs corr_check and page_select first");
  if (ctx->cfg.placement == FKV_PLACE_HOST && ctx->lay.k > 0 && ls.recalled != 3)
    return ctx->fail(FKV_ESTATE, "commit before every head's picked pages were recalled: the page cache would hold unfilled slots");
  ls.parity ^= 1;
  ls.have_prev_q = true;
  ls.have_active = true;
  ls.have_pending = false;
  ls.staged_q = false;
  ls.have_flags = false;
  return FKV_OK;
}

int fkv_commit(fkv_ctx* ctx, int32_t layer) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  return commit_layer(ctx, layer);
}

int fkv_flush(fkv_ctx* ctx) {
  if (!ctx) return FKV_EINVAL;
  return flush_deferred(ctx);
}

int fkv_decode_step(fkv_ctx* ctx, int32_t layer, const void* q_dev, const void* k_new_dev, const void* v_new_dev,
                    float* out_dev, void* compute_stream, void* copy_stream) {
  FKV_CHECK_LAYER(ctx, layer);
  if (!q_dev || !k_new_dev || !v_new_dev || !out_dev) return ctx->fail(FKV_EINVAL, "null argument");
  LayerState& ls = ctx->layers[layer];
  hipStream_t st = static_cast<hipStream_t>(compute_stream);
  hipStream_t cs = static_cast<hipStream_t>(copy_stream);
  if (ls.L >= ctx->cfg.max_ctx) return ctx->fail(FKV_ERANGE, "append beyond max_ctx");
  int rc = FKV_OK;
  if (!ctx->deferred.empty() && (ls.recall_unsubmitted || st != ctx->deferred_st || cs != ctx->deferred_cs)) {
    rc = flush_deferred(ctx);      // this layer's own recall of the last step is still on the list, or the streams changed
    if (rc) return rc;
  }
  rc = wait_recall(ctx, ls, st);
  if (rc) return rc;
  const bool host_pool = ctx->cfg.placement == FKV_PLACE_HOST;
  // everything in one launch when the shape allows it; with the host pool, when the recall is the library's gather into
  // its own page cache (the kernel's attention blocks then fetch a corrected head's missing pages themselves)
  if (!host_pool || (ctx->cfg.recall_mode == FKV_RECALL_GATHER && !ctx->nhd_pool)) {
    if (host_pool && ls.offload_unseen) {      // a page offloaded moments ago may be picked, and missed, already
      FKV_HIP(ctx, hipStreamWaitEvent(st, ls.ev_offload, 0));
      ls.offload_unseen = false;
    }
    const StepIO io = make_step_io(ctx, layer, q_dev, k_new_dev, v_new_dev, nullptr, nullptr);
    LayerIO lio{};
    lio.act_ids = ctx->ids(layer, ls.parity ^ 1);
    lio.part_o = ctx->part_o();
    lio.part_ml = ctx->part_ml();
    lio.max_splits = ctx->lay.max_splits;
    lio.attn_counters = ctx->attn_counters(layer);
    lio.out = out_dev;
    lio.host_pool = host_pool ? ctx->host_pool(layer) : nullptr;
    lio.tagged = ctx->tagged(layer);
    lio.epoch = ls.epoch + 1;
    lio.status = ctx->status(layer);
    lio.attn_epoch_bias = ctx->lose_selection ? 1 : 0;
    lio.launch_grid = &ls.last_grid;
    lio.launch_lds = &ls.last_lds;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (ctx->prof_on && ctx->prof_used + 2 <= ctx->prof_ev.size()) {
      e0 = ctx->prof_ev[ctx->prof_used];
      e1 = ctx->prof_ev[ctx->prof_used + 1];
      (void)hipEventRecord(e0, st);
    }
    if (launch_layer(ctx->dims, io, lio, make_geom(ctx->cfg, ls.L + 1), st)) {
      if (e0) { (void)hipEventRecord(e1, st); ctx->prof_used += 2; }
      rc = after_launch(ctx, "layer kernel");
      if (rc) return rc;
      ls.epoch += 1;
      ls.last_launches = 1;
      ls.step_launches = 1;
      ls.staged_q = ls.have_flags = ls.have_pending = true;
      if (!host_pool) {
        ls.L += 1;
        return commit_layer(ctx, layer);
      }
      rc = after_append(ctx, layer, st, cs);
      if (rc) return rc;
      // The corrected heads' pages are in their slots when the kernel ends.  The other heads' recall, for the next
      // step (Sec. 3.2), goes to the copy stream; it writes only slots that no attention of this step reads.  It is
      // put on the context's list and submitted together with the next layers' (flush_deferred).
      ls.recalled = 3;
      ls.recall_unsubmitted = true;
      ctx->deferred.push_back(layer);
      ctx->deferred_st = st;
      ctx->deferred_cs = cs;
      if ((int)ctx->deferred.size() >= ctx->defer_group || layer == ctx->cfg.n_layers - 1) {
        rc = flush_deferred(ctx);
        if (rc) return rc;
      }
      return commit_layer(ctx, layer);
    }
  }
  // append + correction test + selection for all heads: one launch
  rc = run_step(ctx, layer, ROLE_APPEND | ROLE_CORR | ROLE_SELECT, q_dev, k_new_dev, v_new_dev, nullptr, nullptr,
                ls.L + 1, st);
  if (rc) return rc;
  rc = after_append(ctx, layer, st, cs);
  if (rc) return rc;
  ls.staged_q = ls.have_flags = ls.have_pending = true;
  bool deferred = false;
  if (host_pool) {
    // corrected heads: recall before this step's attention (Sec. 3.3)
    rc = fkv_recall_pending(ctx, layer, FKV_HEADS_FLAGGED, compute_stream);
    if (rc) return rc;
    // other heads: recall for the next step on the copy stream, off the critical path
    // (Sec. 3.2).  It writes only slots that this step's attention does not read, so it may run
    // beside it; it starts behind the corrected heads' recall so that it does not share the
    // host link with the transfer the attention is waiting for.
    if (cs != st) {
      FKV_HIP(ctx, hipEventRecord(ctx->ev_fork, st));
      FKV_HIP(ctx, hipStreamWaitEvent(cs, ctx->ev_fork, 0));
      rc = fkv_recall_pending(ctx, layer, FKV_HEADS_UNFLAGGED, copy_stream);
      if (rc) return rc;
      FKV_HIP(ctx, hipEventRecord(ls.ev_recall, cs));
      forget_waits(ctx, ls.ev_recall);
      ls.recall_event = ls.ev_recall;
      deferred = true;     // the next step of this layer waits for it, not this step's attention
    }
  }
  rc = fkv_sparse_decode_attn(ctx, layer, q_dev, out_dev, FKV_USE_BY_FLAG, compute_stream);
  if (rc) return rc;
  if (host_pool && ctx->nhd_pool) {
    // the literal NHD pool: the pages of Sel(q_i) that are on the GPU already (sink, window, open page, page-cache
    // hits) are converted in place; the missing ones arrive through the streamed recall
    launch_export_nhd(ctx->dims, ctx->pool_desc(layer), ctx->ids(layer, ls.parity ^ 1), ctx->ids(layer, ls.parity),
                      ctx->slots(layer, ls.parity ^ 1), ctx->slots(layer, ls.parity), ctx->flags(layer), FKV_USE_PENDING,
                      ctx->nhd_pool, ctx->nhd_slot_pages, ctx->nhd_slots, make_geom(ctx->cfg, ls.L), st, ctx->miss(layer));
    rc = after_launch(ctx, "NHD export kernel");
    if (rc) return rc;
  }
  if (host_pool && cs == st) {
    rc = fkv_recall_pending(ctx, layer, FKV_HEADS_UNFLAGGED, compute_stream);
    if (rc) return rc;
  }
  ls.recall_outstanding = deferred;
  // step roles (1-4, the recall plan rides with the selection) + attention, and with the host pool the corrected heads' gather
  ls.last_launches = ls.step_launches + 1 + (host_pool ? 1 : 0);
  return commit_layer(ctx, layer);
}

int fkv_test_lose_selection(fkv_ctx* ctx, int32_t on) {
  if (!ctx) return FKV_EINVAL;
  ctx->lose_selection = on != 0;
  return FKV_OK;
}

int fkv_instrument_timestamps(fkv_ctx* ctx, int32_t on) {
  if (!ctx) return FKV_EINVAL;
  ctx->stamp_on = on != 0;
  return FKV_OK;
}

int fkv_profile_enable(fkv_ctx* ctx, int32_t max_launches) {
  if (!ctx) return FKV_EINVAL;
  if (max_launches < 0 || max_launches > (1 << 20)) return ctx->fail(FKV_EINVAL, "max_launches out of range");
  FKV_HIP(ctx, hipDeviceSynchronize());
  ctx->prof_used = 0;
  ctx->prof_on = max_launches > 0;
  while (ctx->prof_ev.size() < (size_t)2 * max_launches) {
    hipEvent_t e;
    FKV_HIP(ctx, hipEventCreate(&e));
    ctx->prof_ev.push_back(e);
  }
  return FKV_OK;
}

int fkv_profile_read(fkv_ctx* ctx, double* total_ms, int32_t* launches) {
  if (!ctx || !total_ms || !launches) return FKV_EINVAL;
  FKV_HIP(ctx, hipDeviceSynchronize());
  double sum = 0.0;
  for (size_t i = 0; i + 1 < ctx->prof_used; i += 2) {
    float ms = 0.f;
    FKV_HIP(ctx, hipEventElapsedTime(&ms, ctx->prof_ev[i], ctx->prof_ev[i + 1]));
    sum += ms;
  }
  *total_ms = sum;
  *launches = (int32_t)(ctx->prof_used / 2);
  ctx->prof_used = 0;
  return FKV_OK;
}

int fkv_profile_attn(fkv_ctx* ctx, const void* q_dev, size_t q_layer_stride, float* out_dev, int32_t reps,
                     void* stream, double* total_ms, int32_t* launches) {
  if (!ctx || !q_dev || !out_dev || !total_ms || !launches || reps < 1) return FKV_EINVAL;
  FKV_FLUSH(ctx);
  hipStream_t st = static_cast<hipStream_t>(stream);
  for (int l = 0; l < ctx->cfg.n_layers; ++l)
    if (ctx->layers[l].L < 1 || !ctx->layers[l].have_active) return ctx->fail(FKV_ESTATE, "every layer needs a context and an active selection");
  hipEvent_t e0, e1;
  FKV_HIP(ctx, hipEventCreate(&e0));
  FKV_HIP(ctx, hipEventCreate(&e1));
  FKV_HIP(ctx, hipDeviceSynchronize());
  FKV_HIP(ctx, hipEventRecord(e0, st));
  int n = 0;
  for (int r = 0; r < reps; ++r) {
    for (int l = 0; l < ctx->cfg.n_layers; ++l, ++n) {
      const LayerState& ls = ctx->layers[l];
      launch_attn(ctx->dims, ctx->pool_desc(l), reinterpret_cast<const uint16_t*>(static_cast<const char*>(q_dev) + q_layer_stride * l),
                  ctx->ids(l, ls.parity ^ 1), ctx->ids(l, ls.parity), ctx->slots(l, ls.parity ^ 1), ctx->slots(l, ls.parity),
                  ctx->flags(l), FKV_USE_ACTIVE, ctx->part_o(), ctx->part_ml(), ctx->lay.max_splits, ctx->attn_counters(l),
                  out_dev, make_geom(ctx->cfg, ls.L), st, nullptr, nullptr, nullptr);
    }
  }
  FKV_HIP(ctx, hipEventRecord(e1, st));
  FKV_HIP(ctx, hipEventSynchronize(e1));
  float ms = 0.f;
  FKV_HIP(ctx, hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  int rc = after_launch(ctx, "attention kernels");
  if (rc) return rc;
  *total_ms = ms;
  *launches = n;
  return FKV_OK;
}

int fkv_profile_select(fkv_ctx* ctx, const void* q_dev, size_t q_layer_stride, int32_t reps, void* stream,
                       double* total_ms, int32_t* launches) {
  if (!ctx || !q_dev || !total_ms || !launches || reps < 1) return FKV_EINVAL;
  FKV_FLUSH(ctx);
  hipStream_t st = static_cast<hipStream_t>(stream);
  for (int l = 0; l < ctx->cfg.n_layers; ++l)
    if (ctx->layers[l].L < 1) return ctx->fail(FKV_ESTATE, "every layer needs a context");
  hipEvent_t e0, e1;
  FKV_HIP(ctx, hipEventCreate(&e0));
  FKV_HIP(ctx, hipEventCreate(&e1));
  FKV_HIP(ctx, hipDeviceSynchronize());
  FKV_HIP(ctx, hipEventRecord(e0, st));
  int n = 0;
  for (int r = 0; r < reps; ++r) {
    for (int l = 0; l < ctx->cfg.n_layers; ++l) {
      const StepIO io = make_step_io(ctx, l, static_cast<const char*>(q_dev) + q_layer_stride * l, nullptr, nullptr, nullptr, nullptr);
      n += launch_step(ctx->dims, ROLE_SELECT, io, make_geom(ctx->cfg, ctx->layers[l].L), st);
    }
  }
  FKV_HIP(ctx, hipEventRecord(e1, st));
  FKV_HIP(ctx, hipEventSynchronize(e1));
  float ms = 0.f;
  FKV_HIP(ctx, hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  int rc = after_launch(ctx, "step kernels");
  if (rc) return rc;
  *total_ms = ms;
  *launches = n;
  return FKV_OK;
}

int fkv_profile_launch_floor(fkv_ctx* ctx, int32_t layer, int32_t reps, void* stream, double* total_ms,
                             int32_t* grid, int32_t* lds_bytes) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  if (!total_ms || reps < 1) return ctx->fail(FKV_EINVAL, "bad argument");
  const LayerState& ls = ctx->layers[layer];
  if (ls.last_launches != 1 || ls.last_grid < 1) return ctx->fail(FKV_ESTATE, "the layer's last step was not a single launch");
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipEvent_t e0, e1;
  FKV_HIP(ctx, hipEventCreate(&e0));
  FKV_HIP(ctx, hipEventCreate(&e1));
  FKV_HIP(ctx, hipDeviceSynchronize());
  if (!launch_floor(ls.last_grid, ls.last_lds, 4, st)) return ctx->fail(FKV_EHIP, "empty kernel refused its LDS size");
  FKV_HIP(ctx, hipEventRecord(e0, st));
  launch_floor(ls.last_grid, ls.last_lds, reps, st);
  FKV_HIP(ctx, hipEventRecord(e1, st));
  FKV_HIP(ctx, hipEventSynchronize(e1));
  float ms = 0.f;
  FKV_HIP(ctx, hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  int rc = after_launch(ctx, "empty kernels");
  if (rc) return rc;
  *total_ms = ms;
  if (grid) *grid = ls.last_grid;
  if (lds_bytes) *lds_bytes = (int32_t)ls.last_lds;
  return FKV_OK;
}

int fkv_debug_read(fkv_ctx* ctx, int32_t layer, int32_t what, void* host_out, size_t bytes) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  if (!host_out) return ctx->fail(FKV_EINVAL, "null output");
  const fkv_config& c = ctx->cfg;
  const LayerState& ls = ctx->layers[layer];
  const size_t kk = ctx->lay.k;
  const void* src = nullptr;
  size_t n = 0;
  switch (what) {
    case FKV_DBG_SUMMARIES:   src = ctx->summ(layer); n = (size_t)c.batch * c.n_kv_heads * 2 * ctx->lay.max_pages * D * 2; break;
    case FKV_DBG_WEIGHTS:     src = ctx->P(); n = (size_t)c.batch * c.n_q_heads * ctx->lay.max_pages * 4; break;
    case FKV_DBG_SCORES:      src = ctx->score(); n = (size_t)c.batch * c.n_kv_heads * ctx->lay.max_pages * 4; break;
    case FKV_DBG_ACTIVE_IDS:  src = ctx->ids(layer, ls.parity ^ 1); n = (size_t)c.batch * c.n_kv_heads * kk * 4; break;
    case FKV_DBG_PENDING_IDS: src = ctx->ids(layer, ls.parity); n = (size_t)c.batch * c.n_kv_heads * kk * 4; break;
    case FKV_DBG_FLAGS:       src = ctx->flags(layer); n = (size_t)c.batch * c.n_kv_heads; break;
    case FKV_DBG_COSINE:      src = ctx->cosine(layer); n = (size_t)c.batch * c.n_q_heads * 8; break;
    case FKV_DBG_TSTAMP:      src = ctx_base_tstamp(ctx); n = 64 * 8; break;
    case FKV_DBG_MISS: {
      n = (size_t)c.batch * c.n_kv_heads * (1 + kk) * 4;
      if (bytes < n) return ctx->fail(FKV_EINVAL, "output buffer too small");
      FKV_HIP(ctx, hipDeviceSynchronize());
      std::vector<int32_t> tmp((size_t)c.batch * c.n_kv_heads * (1 + 3 * kk));
      FKV_HIP(ctx, hipMemcpy(tmp.data(), ctx->miss(layer), tmp.size() * 4, hipMemcpyDeviceToHost));
      int32_t* o = static_cast<int32_t*>(host_out);
      for (int h = 0; h < c.batch * c.n_kv_heads; ++h) {
        const int32_t* mh = tmp.data() + (size_t)h * (1 + 3 * kk);
        o[(size_t)h * (1 + kk)] = mh[0];
        for (size_t i = 0; i < kk; ++i) o[(size_t)h * (1 + kk) + 1 + i] = (int32_t)i < mh[0] ? mh[1 + i] : -1;
      }
      return FKV_OK;
    }
    default: return ctx->fail(FKV_EINVAL, "unknown debug item");
  }
  if (bytes < n) return ctx->fail(FKV_EINVAL, "output buffer too small");
  FKV_HIP(ctx, hipDeviceSynchronize());
  if (n) FKV_HIP(ctx, hipMemcpy(host_out, src, n, hipMemcpyDeviceToHost));
  return FKV_OK;
}

int fkv_debug_read_page(fkv_ctx* ctx, int32_t layer, int32_t request, int32_t kv_head, int32_t page, int32_t where, void* host_out) {
  FKV_CHECK_LAYER(ctx, layer);
  FKV_FLUSH(ctx);
  const fkv_config& c = ctx->cfg;
  if (!host_out) return ctx->fail(FKV_EINVAL, "null output");
  if (request < 0 || request >= c.batch || kv_head < 0 || kv_head >= c.n_kv_heads) return ctx->fail(FKV_ERANGE, "request or head out of range");
  const LayerState& ls = ctx->layers[layer];
  if (page < 0 || page >= (ls.L + PG - 1) / PG) return ctx->fail(FKV_ERANGE, "page beyond the cached context");
  FKV_HIP(ctx, hipDeviceSynchronize());
  const size_t head = (size_t)request * c.n_kv_heads + kv_head;
  const PoolDesc pd = ctx->pool_desc(layer);
  const uint16_t* unit = nullptr;
  if (where == 0) {
    if (c.placement != FKV_PLACE_HBM) return ctx->fail(FKV_ESTATE, "no HBM store in host placement");
    unit = pd.pool + (head * pd.units_per_head + page) * UNIT_ELEMS;
  } else if (where == 1) {
    if (c.placement != FKV_PLACE_HOST) return ctx->fail(FKV_ESTATE, "no host pool in HBM placement");
    unit = ctx->host_pool(layer) + (head * ctx->lay.max_pages + page) * UNIT_ELEMS;
  } else if (where == 2 || where == 3) {
    if (c.placement != FKV_PLACE_HOST) return ctx->fail(FKV_ESTATE, "no page cache in HBM placement");
    const size_t kk = ctx->lay.k;
    const int half = where == 2 ? ls.parity ^ 1 : ls.parity;
    std::vector<int32_t> idv(kk), slv(kk);
    FKV_HIP(ctx, hipMemcpy(idv.data(), ctx->ids(layer, half) + head * kk, kk * 4, hipMemcpyDeviceToHost));
    FKV_HIP(ctx, hipMemcpy(slv.data(), ctx->slots(layer, half) + head * kk, kk * 4, hipMemcpyDeviceToHost));
    int slot = -1;
    for (size_t i = 0; i < kk; ++i) if (idv[i] == page) slot = slv[i];
    if (slot < 0) return ctx->fail(FKV_ERANGE, "page is not in that selection");
    unit = pd.pool + (head * pd.units_per_head + pd.sel_base + slot) * UNIT_ELEMS;
  } else {
    return ctx->fail(FKV_EINVAL, "bad where");
  }
  launch_read_page(unit, ctx->dbg_page(), nullptr);
  int rc = after_launch(ctx, "read_page kernel");
  if (rc) return rc;
  FKV_HIP(ctx, hipDeviceSynchronize());
  FKV_HIP(ctx, hipMemcpy(host_out, ctx->dbg_page(), UNIT_BYTES, hipMemcpyDeviceToHost));
  return FKV_OK;
}

}  // extern "C"
