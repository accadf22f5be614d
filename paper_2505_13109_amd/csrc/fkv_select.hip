// The "step" kernel (token append, correction test, page weights, and -- in its last scoring
// block per KV head or in a launch of its own -- the top-k selection), the one-launch layer kernel
// (the step roles plus the attention blocks), and the host-side rules that size their launches.
// The roles themselves are in fkv_step_dev.h, attention in fkv_attn_dev.h.
#include "fkv_step_dev.h"
#include "fkv_attn_dev.h"

#pragma clang fp contract(off)

namespace fkv {

// ---------------------------------------------------------------------------------
// the kernel: 1-D grid, [append blocks][corr blocks][scoring blocks], each set present
// only if its role bit is set; heads = batch * n_kv.
// ---------------------------------------------------------------------------------
template <int DT, int G>
__global__ __launch_bounds__(STEP_THREADS, STEP_THREADS <= 256 ? 2 : 1) void step_kernel(StepArgs a) {
  extern __shared__ uint32_t dyn_lds[];              // selection: n_cand keys, then G x n_cand weights
  step_roles<DT, G, false>(a, blockIdx.x, dyn_lds);
}

// The scan of the bandwidth-bound regime: append, correction test and page weights only (the selection has
// a launch of its own there), in 256-thread blocks of one 64-page chunk each.  Measured on the scan alone
// (256 heads x 992 pages, 130 MB; a plain read of the same bytes takes 22.1 us = 5.9 TB/s on this machine):
// 23.9 us in this shape against 25.7 us with 512-thread blocks of 128 pages -- the smaller block leaves
// the unit's slots in finer pieces, so that more blocks are in different phases (loading, computing,
// draining) at any time; blocks that take several chunks, pipelined or not, are slower than either.
constexpr int SCAN_WAVES = 4, SCAN_PASSES = 4;
template <int DT, int G>
__global__ __launch_bounds__(SCAN_WAVES * 64) void scan_kernel(StepArgs a) {
  const int heads = a.batch * a.n_kv;
  int bid = blockIdx.x;
  if (a.roles & ROLE_APPEND) {
    if (bid < heads) { append_role<DT>(a, bid); return; }
    bid -= heads;
  }
  if (a.roles & ROLE_CORR) {
    if (bid < heads) { corr_role<DT, G, SCAN_WAVES>(a, bid); return; }
    bid -= heads;
  }
  score_role<DT, G, SCAN_WAVES>(a, bid / a.blocks_per_head, bid % a.blocks_per_head);
}

// Dynamic LDS above the default 64 KiB per block has to be granted per kernel function.
// Returns false if the device refuses (the caller then keeps only the keys in LDS).
template <int DT, int G>
static bool raise_lds(size_t lds) {
  static size_t granted = 0;
  if (lds <= granted) return true;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(&step_kernel<DT, G>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  granted = lds;
  return true;
}

// The selection's LDS (keys + staged weights) is allocated for every block of a launch.  When
// it is small and the launch is at most one round of blocks, the selection rides in the scoring
// launch (its last block per head runs it); otherwise scoring runs without it and a second
// launch of one block per head selects.
constexpr size_t kLdsPerUnit = 150 * 1024;   // of the 160 KiB of a compute unit
constexpr int kComputeUnits = 256;
constexpr int kFuseMaxBlocks = kComputeUnits;       // launches up to this size run the selection in their last scoring blocks
constexpr int kLayerMaxBlocks = 4 * kComputeUnits;  // shapes up to this size take the one-launch layer kernel
// experiment builds only (see knob()): chunks per scoring block, selection inside the scoring launch
// (0 never, 1 always), passes a scoring block makes; the defaults choose from the shape
static const int g_chunks_per_block = knob("FKV_SCORE_CHUNKS", 0);
static const int g_fuse_mode = knob("FKV_FUSE_SELECT", -1);
static const int g_min_passes = knob("FKV_LAYER_PASSES", 0);
static const bool g_scan_kernel = knob("FKV_NO_SCAN_KERNEL", 0) == 0;   // 1: scans stay in 512-thread step_kernel blocks
// may every block of a `grid`-block launch carry `lds` bytes without starving the scoring blocks?
static bool lds_fits_launch(size_t lds, int grid) {
  int per_unit = (grid + kComputeUnits - 1) / kComputeUnits;   // blocks a unit should hold at once
  if (per_unit < 1) per_unit = 1;
  if (per_unit > 4) per_unit = 4;
  return lds * per_unit <= kLdsPerUnit;
}

struct WidePlan { const Dims* d; const StepIO* io; bool ok; int B, slice; };

template <int DT, int G>
static int launch_step_g(StepArgs& a, int grid, int heads, size_t lds_staged, size_t lds_keys, hipStream_t st, const WidePlan& wp) {
  constexpr size_t kDefaultLimit = 64 * 1024 - 8 * 1024;   // minus this kernel's static LDS, rounded up
  const bool select = (a.roles & ROLE_SELECT) != 0;
  size_t lds = lds_staged;
  a.staged = lds_staged > lds_keys ? 1 : 0;
  if (select && a.staged && lds > kDefaultLimit && !raise_lds<DT, G>(lds)) {
    lds = lds_keys;
    a.staged = 0;
  }
  if (select && !a.staged && lds > kDefaultLimit) (void)raise_lds<DT, G>(lds);
  // In a launch of many rounds the scoring blocks should end the moment their weights are on the
  // way: waiting for the stores' acknowledgement and the counter (what the fused selection needs)
  // would hold the unit's slots for several memory round trips per block.
  a.fuse_select = (select && lds_fits_launch(lds, grid) && (g_fuse_mode < 0 ? grid <= kFuseMaxBlocks : g_fuse_mode == 1)) ? 1 : 0;
  a.select_only = 0;
  // a long candidate list whose selection has its own launch anyway is spread over several blocks per head
  const bool wide = wp.ok && select && !a.fuse_select;
  a.bmax = wide ? wp.io->bmax : nullptr;
  a.bmax_stride = wp.io->bmax_stride;
  // the recall plan rides at the end of the selecting block's LDS; a spread selection is followed by the plan kernel
  const bool plan = select && a.plan_new_slots != nullptr;
  const size_t plan_bytes = plan ? plan_lds_ints(a.k) * sizeof(int32_t) : 0;
  a.plan_lds_off = (int)((lds - plan_bytes) / sizeof(uint32_t));
  int32_t* const plan_slots = a.plan_new_slots;
  auto plan_after_wide = [&]() -> int {
    if (!plan) return 0;
    launch_plan(*wp.d, a.ids, a.plan_act_ids, a.plan_act_slots, plan_slots, a.plan_miss, a.g.n_full, st);
    return 1;
  };
  if (wide) a.plan_new_slots = nullptr;
  if (select && !a.fuse_select && g_scan_kernel) {
    // the selection does not ride along: the roles go to the scan kernel, one 64-page chunk per 256-thread block
    StepArgs sa = a;
    sa.passes = SCAN_PASSES;
    sa.blocks_per_head = a.g.n_cand > 0 ? (a.g.n_cand + SCAN_WAVES * 4 * SCAN_PASSES - 1) / (SCAN_WAVES * 4 * SCAN_PASSES) : 1;
    int sgrid = heads * sa.blocks_per_head;
    if (sa.roles & ROLE_APPEND) sgrid += heads;
    if (sa.roles & ROLE_CORR) sgrid += heads;
    const bool fits = !wide || sa.blocks_per_head <= sa.bmax_stride;
    if (fits) {
      scan_kernel<DT, G><<<sgrid, SCAN_WAVES * 64, 0, st>>>(sa);
      if (wide) {
        launch_wide_select(*wp.d, *wp.io, a.g, wp.B, wp.slice, sa.blocks_per_head, st);
        return 3 + plan_after_wide();
      }
      a.select_only = 1;
      step_kernel<DT, G><<<heads, STEP_THREADS, lds, st>>>(a);
      return 2;
    }
  }
  step_kernel<DT, G><<<grid, STEP_THREADS, a.fuse_select ? lds : 0, st>>>(a);
  if (wide) {
    launch_wide_select(*wp.d, *wp.io, a.g, wp.B, wp.slice, a.blocks_per_head, st);
    return 3 + plan_after_wide();
  }
  if (select && !a.fuse_select) {
    a.select_only = 1;
    step_kernel<DT, G><<<heads, STEP_THREADS, lds, st>>>(a);
    return 2;
  }
  return 1;
}

template <int DT>
static int launch_step_dt(StepArgs& a, int G, int grid, int heads, size_t lds_staged, size_t lds_keys, hipStream_t st, const WidePlan& wp) {
  switch (G) {
#define FKV_CASE(GG) case GG: return launch_step_g<DT, GG>(a, grid, heads, lds_staged, lds_keys, st, wp);
    FKV_CASE(1) FKV_CASE(2) FKV_CASE(3) FKV_CASE(4) FKV_CASE(5) FKV_CASE(6) FKV_CASE(7) FKV_CASE(8)
#undef FKV_CASE
    default: return 0;
  }
}

static void fill_step_args(const Dims& d, int roles, const StepIO& io, Geom g, int passes, bool roomy, StepArgs& a,
                           int& grid, size_t& lds_staged, size_t& lds_keys, int chunks_per_block = 1) {
  a = StepArgs{};
  a.roles = roles;
  a.batch = d.batch; a.n_q = d.n_q; a.n_kv = d.n_kv; a.k = d.k; a.max_pages = d.max_pages;
  a.g = g;
  a.pd = io.pd; a.summ = io.summ; a.k_new = io.k_new; a.v_new = io.v_new;
  a.q = io.q; a.q_prev = io.q_prev; a.q_stage = io.q_stage; a.have_prev = io.have_prev; a.tau = io.tau;
  a.corr_pool = d.corr_pool; a.sel_pool = d.sel_pool;
  a.flags = io.flags; a.flags_user = io.flags_user; a.cosine = io.cosine;
  a.P = io.P; a.score = io.score; a.ids = io.ids; a.ids_user = io.ids_user; a.counters = io.counters; a.tstamp = io.tstamp;
  const int heads = d.batch * d.n_kv;
  a.passes = passes;
  const int chunks = g.n_cand > 0 ? (g.n_cand + PAGES_PER_PASS * passes - 1) / (PAGES_PER_PASS * passes) : 1;
  a.blocks_per_head = (chunks + chunks_per_block - 1) / chunks_per_block;
  grid = 0;
  lds_staged = lds_keys = 0;
  if (roles & ROLE_APPEND) grid += heads;
  if (roles & ROLE_CORR) grid += heads;
  if (roles & ROLE_SELECT) {
    grid += heads * a.blocks_per_head;
    const size_t n = (size_t)(g.n_cand > 0 ? g.n_cand : 1);
    lds_keys = n * sizeof(uint32_t);
    lds_staged = n * (1 + d.G) * sizeof(uint32_t);
    if (io.plan_new_slots) {
      a.plan_act_ids = io.plan_act_ids; a.plan_act_slots = io.plan_act_slots;
      a.plan_new_slots = io.plan_new_slots; a.plan_miss = io.plan_miss;
    }
    const size_t plan_bytes = io.plan_new_slots ? plan_lds_ints(d.k) * sizeof(int32_t) : 0;
    if (lds_staged + plan_bytes + 8192 > (size_t)d.max_lds) lds_staged = lds_keys;   // cannot fit: do not even ask
    if (n <= (size_t)regs_candidates(d.G, roomy)) lds_staged = lds_keys;   // few enough to stay in registers
    lds_staged += plan_bytes;                      // the recall plan's LDS follows the selection's
    lds_keys += plan_bytes;
  }
}

// The roles of one launch run concurrently.  That is safe because the page being appended to
// is not a candidate -- except with an empty window, when the token that fills a page makes
// that very page a candidate in the same step.
static bool append_races_selection(int roles, const Geom& g) {
  return (roles & ROLE_APPEND) && (roles & ROLE_SELECT) && g.r == 0 && g.n_win == 0 && g.n_cand > 0;
}

int launch_step(const Dims& d, int roles, const StepIO& io, Geom g, hipStream_t st) {
  if (d.k == 0) roles &= ~ROLE_SELECT;
  if (roles == 0) return 0;
  int launches = 0;
  if (append_races_selection(roles, g)) {      // then the append gets a launch of its own first
    launches += launch_step(d, ROLE_APPEND, io, g, st);
    roles &= ~ROLE_APPEND;
  }
  StepArgs a;
  int grid;
  size_t lds_staged, lds_keys;
  // A scoring block lives for one memory round trip whatever it loads, so big scans get fewer
  // blocks with more pages in flight each, as long as a few blocks per compute unit remain.
  int passes = g_min_passes > 0 ? g_min_passes : 1;
  if (g_min_passes <= 0 && (roles & ROLE_SELECT))
    while (passes < SCORE_PASSES &&
           (long)d.batch * d.n_kv * ((g.n_cand + PAGES_PER_PASS * passes * 2 - 1) / (PAGES_PER_PASS * passes * 2)) >= 4 * kComputeUnits)
      passes *= 2;
  // ... and beyond a few blocks per unit, a block takes several chunks in turn: a block's fixed cost
  // (dispatch, the query loads, the drain of its stores) is what is left to save once the scan
  // streams.  (Prefetching the next chunk into a second register set was measured and dropped: the
  // registers it takes halve the blocks a unit holds, and two blocks that load and compute in turn
  // stream faster than one that overlaps its own loads.)
  int chunks_per_block = g_chunks_per_block > 0 ? g_chunks_per_block : 1;
  if (g_chunks_per_block <= 0 && (roles & ROLE_SELECT)) {
    const long blocks = (long)d.batch * d.n_kv * ((g.n_cand + PAGES_PER_PASS * passes - 1) / (PAGES_PER_PASS * passes));
    while (chunks_per_block < 16 && blocks / chunks_per_block > 4 * kComputeUnits) chunks_per_block *= 2;
  }
  fill_step_args(d, roles, io, g, passes, false, a, grid, lds_staged, lds_keys, chunks_per_block);
  WidePlan wp{&d, &io, false, 0, 0};
  wp.ok = (roles & ROLE_SELECT) && io.bmax && a.blocks_per_head <= io.bmax_stride && knob("FKV_NO_WIDE_SELECT", 0) == 0 && wide_plan(d, g, &wp.B, &wp.slice);
  if (d.dtype == 0) launches += launch_step_dt<0>(a, d.G, grid, d.batch * d.n_kv, lds_staged, lds_keys, st, wp);
  else              launches += launch_step_dt<1>(a, d.G, grid, d.batch * d.n_kv, lds_staged, lds_keys, st, wp);
  return launches;
}

// ---------------------------------------------------------------------------------
// The whole layer-step in ONE launch (KV in HBM, small selections): the step roles followed by
// the attention blocks.  In a step without correction the two chains do not depend on each
// other -- attention reads the previous step's page ids, takes the new token from the step's
// inputs and redoes the (tiny) correction test itself -- so they overlap; the attention blocks
// of a corrected head wait for that head's selection, made by blocks with lower indices.
// ---------------------------------------------------------------------------------
struct LayerArgs {
  StepArgs s;
  AttnArgs at;
  int attn_block0;     // index of the first attention block
};

template <int DT, int G, bool HOSTPOOL>
__global__ __launch_bounds__(STEP_THREADS, STEP_THREADS <= 256 ? 2 : 1) void layer_kernel(LayerArgs a) {
  extern __shared__ uint32_t dyn_lds[];
  if ((int)blockIdx.x < a.attn_block0) {
    step_roles<DT, G, true>(a.s, blockIdx.x, dyn_lds);
    return;
  }
  const int ab = blockIdx.x - a.attn_block0, heads = a.s.batch * a.s.n_kv;
  const int head = ab % heads, split = ab / heads;
  attn_block<DT, STEP_WAVES, HOSTPOOL>(a.at, split, head % a.s.n_kv, head / a.s.n_kv, reinterpret_cast<float*>(dyn_lds));
}

// experiment builds only: 1 = always separate launches, 0 = one launch whenever it fits
static const bool g_no_layer_kernel = knob("FKV_NO_LAYER_KERNEL", -1) == 1;
static const bool g_layer_always = knob("FKV_NO_LAYER_KERNEL", -1) == 0;

template <int DT, int G, bool HOSTPOOL>
static bool launch_layer_gh(const LayerArgs& a, int grid, size_t lds, hipStream_t st) {
  static size_t granted = 48 * 1024;      // dynamic LDS beyond the default has to be granted per function
  if (lds > granted) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&layer_kernel<DT, G, HOSTPOOL>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
      (void)hipGetLastError();
      return false;
    }
    granted = lds;
  }
  layer_kernel<DT, G, HOSTPOOL><<<grid, STEP_THREADS, lds, st>>>(a);
  return true;
}
template <int DT, int G>
static bool launch_layer_g(const LayerArgs& a, int grid, size_t lds, hipStream_t st) {
  return a.at.host_pool ? launch_layer_gh<DT, G, true>(a, grid, lds, st) : launch_layer_gh<DT, G, false>(a, grid, lds, st);
}

bool launch_layer(const Dims& d, const StepIO& io, const LayerIO& lio, Geom g, hipStream_t st) {
  const int roles = ROLE_APPEND | ROLE_CORR | ROLE_SELECT;
  if (g_no_layer_kernel || d.k == 0 || append_races_selection(roles, g)) return false;
  if (io.pd.placement != 0) {
    // KV in a host pool: the selecting blocks make the recall plan, the attention blocks of a corrected head fetch its
    // missing pages themselves; the tagged words have to hold a page id and a slot
    if (!io.plan_new_slots || !lio.host_pool || d.max_pages > TAGGED_MAX_PAGES || 2 * d.k > TAGGED_MAX_SLOTS) return false;
  }
  {   // a candidate list long enough for the selection to be spread over several blocks takes the separate launches
    int wb, ws;
    if (io.bmax && knob("FKV_NO_WIDE_SELECT", 0) == 0 && wide_plan(d, g, &wb, &ws)) return false;
  }
  LayerArgs a{};
  int grid = 0;
  size_t lds = 0;
  // the launch with scoring blocks that make `passes` passes; does every block's LDS fit?
  auto plan = [&](int passes) -> bool {
    size_t lds_staged, lds_keys;
    fill_step_args(d, roles, io, g, passes, true, a.s, grid, lds_staged, lds_keys);
    a.s.staged = lds_staged > lds_keys ? 1 : 0;
    a.s.fuse_select = 1;
    a.s.select_only = 0;
    a.s.tagged = lio.tagged;
    a.s.epoch = lio.epoch;
    a.s.plan_lds_off = (int)((lds_staged - (a.s.plan_new_slots ? plan_lds_ints(d.k) * sizeof(int32_t) : 0)) / sizeof(uint32_t));
    const int heads = d.batch * d.n_kv;
    const int n_att = g.n_sink + d.k + g.n_win + (g.r > 0 ? 1 : 0);
    AttnArgs& at = a.at;
    at.pd = io.pd; at.q = io.q; at.act_ids = lio.act_ids; at.new_ids = io.ids;
    at.act_slots = io.plan_act_slots; at.new_slots = io.plan_new_slots;       // (null with the KV in HBM)
    at.host_pool = lio.host_pool; at.max_pages = d.max_pages;
    at.flags = io.flags; at.use = 2; at.part_o = lio.part_o; at.part_ml = lio.part_ml; at.max_splits = lio.max_splits;
    at.pps = attn_pages_per_block(n_att, heads, lio.max_splits, STEP_WAVES);
    at.n_splits = (n_att + at.pps - 1) / at.pps;
    at.counters = lio.attn_counters; at.out = lio.out; at.g = g;
    at.n_q = d.n_q; at.n_kv = d.n_kv; at.G = d.G; at.k = d.k; at.tstamp = io.tstamp;
    at.fused = 1; at.q_prev = io.q_prev; at.have_prev = io.have_prev; at.tau = io.tau; at.corr_pool = d.corr_pool;
    at.k_new = io.k_new; at.v_new = io.v_new; at.tagged = lio.tagged; at.epoch = lio.epoch + lio.attn_epoch_bias; at.status = lio.status;
    a.attn_block0 = grid;
    grid += heads * at.n_splits;
    const size_t lds_attn = (size_t)STEP_WAVES * (32 + d.G * D) * sizeof(float);
    lds = lds_staged > lds_attn ? lds_staged : lds_attn;
    return lds_fits_launch(lds, grid);
  };
  // The kernel's registers allow one block per compute unit at a time, so a launch runs in
  // ceil(blocks / units) rounds, and blocks of a later round (attention comes last) queue behind
  // the scoring blocks.  Take the passes per scoring block that give the fewest rounds -- one, the
  // whole launch resident at once, where the shape allows -- and among those the fewest passes
  // (most blocks); fatter scoring blocks are also what lets a big selection's LDS fit at all.
  int chosen = 0, best_rounds = 0;
  for (int passes = g_min_passes > 0 ? g_min_passes : 1; passes <= SCORE_PASSES; passes *= 2) {
    if (!plan(passes)) continue;
    const int rounds = (grid + kComputeUnits - 1) / kComputeUnits;
    if (!chosen || rounds < best_rounds) { chosen = passes; best_rounds = rounds; }
    if (g_min_passes > 0) break;
  }
  // Big shapes are bandwidth-bound, not latency-bound: there the separate kernels, with their
  // smaller register footprints and blocks that never wait, stream faster than this one.
  const bool fits = chosen != 0 && plan(chosen) && (grid <= kLayerMaxBlocks || g_layer_always);
  if (!fits) return false;                                 // big selections keep their own launches
  if (lio.launch_grid) *lio.launch_grid = grid;
  if (lio.launch_lds) *lio.launch_lds = lds;
  switch (d.G) {
#define FKV_CASE(GG) case GG: return d.dtype == 0 ? launch_layer_g<0, GG>(a, grid, lds, st) : launch_layer_g<1, GG>(a, grid, lds, st);
    FKV_CASE(1) FKV_CASE(2) FKV_CASE(3) FKV_CASE(4) FKV_CASE(5) FKV_CASE(6) FKV_CASE(7) FKV_CASE(8)
#undef FKV_CASE
    default: return false;
  }
  return true;
}

// ---------------------------------------------------------------------------------
// The cost of a launch as such: a kernel of the same shape whose blocks return at once.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(STEP_THREADS) void floor_kernel(uint32_t* sink) {
  extern __shared__ uint32_t dyn_lds[];
  if (sink) *sink = dyn_lds[0];             // never taken: keeps the LDS allocation in the kernel
}

bool launch_floor(int grid, size_t lds, int reps, hipStream_t st) {
  static size_t granted = 48 * 1024;
  if (lds > granted) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&floor_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) {
      (void)hipGetLastError();
      return false;
    }
    granted = lds;
  }
  for (int r = 0; r < reps; ++r) floor_kernel<<<grid, STEP_THREADS, lds, st>>>(nullptr);
  return true;
}

}  // namespace fkv
