// Internal declarations shared by the host API and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

namespace fkv {

// Dispatch overrides for experiments (sweeps of tile and launch shapes).  They are read from the
// environment only in a build with -DFKV_EXPERIMENT_KNOBS; the product library has none.
inline int knob(const char* name, int dflt) {
#ifdef FKV_EXPERIMENT_KNOBS
  const char* e = getenv(name);
  return e ? atoi(e) : dflt;
#else
  (void)name;
  return dflt;
#endif
}

constexpr int D = 128;            // head_dim
constexpr int PG = 32;            // page size p
constexpr int UNIT_ELEMS = 2 * PG * D;        // K page then V page of one (page, KV head)
constexpr int UNIT_BYTES = UNIT_ELEMS * 2;    // 16 KiB, the contiguous recall unit (Sec. 4.2)
constexpr int MAX_G = 8;

// Geometry of the budget at the current context length (Sec. 2.1: B, S, W).
struct Geom {
  int L;        // tokens cached, the appended one included
  int n_full;   // full pages
  int r;        // tokens in the open page
  int n_sink;   // sink pages [0, n_sink)
  int n_win;    // window pages [n_full - n_win, n_full)
  int cand_lo;  // candidate pages [cand_lo, cand_lo + n_cand)
  int n_cand;
  int k_eff;    // pages picked per KV head = min(k, n_cand)
};

// Where a KV head's pages live in HBM.  Unit u of head (b, m) starts at
// pool + ((b * n_kv + m) * units_per_head + u) * UNIT_ELEMS.
struct PoolDesc {
  uint16_t* pool;
  int units_per_head;
  int placement;     // 0: unit = page id.  1: sink page i -> unit i, window/open page j -> ring_base + j % n_ring,
  int ring_base;     //    picked page in slot s -> sel_base + s
  int n_ring;
  int sel_base;
};

// ---- element offsets inside a unit -------------------------------------
// K page: [s*2+mb (8)][kb (4)][m (16)][e (8)] with channel = (s*4+kb)*8 + e, token = mb*16 + m.
// Each group of 512 elements (1 KiB) is one operand load of the 16x16x32 MFMA
// computing S^T = K Q^T: lane (kb*16 + m) reads 8 consecutive channels of token m.
__host__ __device__ inline int k_elem_off(int t, int ch) {
  int s = ch >> 5, kb = (ch >> 3) & 3, e = ch & 7, mb = t >> 4, m = t & 15;
  return ((((s * 2 + mb) * 4 + kb) * 16 + m) * 8) + e;
}
// V page: [cb (8)][kb (4)][m (16)][e (8)] with channel = cb*16 + m and
// token = (e < 4) ? kb*4 + e : 16 + kb*4 + (e - 4): the token order in which the
// S^T accumulators of a lane come out, so P feeds the second MFMA from registers.
__host__ __device__ inline int v_elem_off(int t, int ch) {
  int cb = ch >> 4, m = ch & 15, hi = t >> 4, kb = (t & 15) >> 2, e = (t & 3) + 4 * hi;
  return PG * D + (((cb * 4 + kb) * 16 + m) * 8) + e;
}

// ---- launch wrappers (defined in the kernel files) ----------------------
struct Dims { int batch, n_q, n_kv, G, k, max_pages, dtype, max_lds, sel_pool, corr_pool; };

// the fused step kernel: roles are OR-ed
constexpr int ROLE_APPEND = 1, ROLE_CORR = 2, ROLE_SELECT = 4;
struct StepIO {
  PoolDesc pd; uint16_t* summ; const uint16_t* k_new; const uint16_t* v_new;      // append
  const uint16_t* q; const uint16_t* q_prev; uint16_t* q_stage; int have_prev; float tau;
  uint8_t* flags; uint8_t* flags_user; double* cosine;                               // correction test
  float* P; float* score; int32_t* ids; int32_t* ids_user; int* counters;            // selection
  long long* tstamp;                                                                 // debug timestamps or null
  // scratch of a selection spread over several blocks per head (all may be null: then it is never spread)
  float* bmax; int bmax_stride; float* hmax; unsigned long long* zsum; uint32_t* cand_key; int32_t* cand_id; int* wide_counters;
  // KV in a host pool (else all null): a launch with ROLE_SELECT also makes the recall plan of the new selection --
  // ACTIVE ids and slots in, PENDING slots and miss lists out
  const int32_t* plan_act_ids; const int32_t* plan_act_slots; int32_t* plan_new_slots; int32_t* plan_miss;
};
constexpr int WIDE_MAX_SLICES = 16;       // most blocks that share one head's selection
bool wide_plan(const Dims& d, const Geom& g, int* B, int* slice);
void launch_wide_select(const Dims& d, const StepIO& io, Geom g, int B, int slice, int n_score_blocks, hipStream_t st);
int launch_step(const Dims& d, int roles, const StepIO& io, Geom g, hipStream_t st);   // returns the launches made
// the whole layer-step (step roles + attention) in one launch; false if this shape or placement
// has to take the separate launches
struct LayerIO {
  const int32_t* act_ids; float* part_o; float* part_ml; int max_splits; int* attn_counters; float* out;
  const uint16_t* host_pool;                 // KV in a host pool: this layer's pool (corrected heads fetch their missing pages from it)
  unsigned long long* tagged; int epoch; int* status;   // tagged: [heads][k] epoch-tagged copies of the picked ids
  int attn_epoch_bias;                       // 0; a test of the bounded wait makes attention wait for an epoch that never comes
  int* launch_grid; size_t* launch_lds;      // out (may be null): shape of the launch that was made
};
// `reps` launches of a kernel that does nothing, with the given grid, 512 threads and dynamic LDS
bool launch_floor(int grid, size_t lds, int reps, hipStream_t st);
bool launch_layer(const Dims& d, const StepIO& io, const LayerIO& lio, Geom g, hipStream_t st);
int attn_pages_per_block(int n_att, int heads, int max_splits, int nw);
void launch_load_prefix(const Dims& d, const PoolDesc& pd, uint16_t* summ, uint16_t* host_pool,
                        const uint16_t* K, const uint16_t* V, int n_tokens, Geom g, hipStream_t st);
void launch_summary_recompute(const Dims& d, const PoolDesc& pd, uint16_t* summ, int first_page,
                              int n_pages, Geom g, hipStream_t st);
void launch_offload(const Dims& d, const PoolDesc& pd, uint16_t* host_pool, int page, hipStream_t st);
// new_ids is read and, where an id is not a full page (id < 0 or id >= n_full), rewritten to -1
void launch_plan(const Dims& d, int32_t* new_ids, const int32_t* act_ids, const int32_t* act_slots,
                 int32_t* new_slots, int32_t* miss, int n_full, hipStream_t st);
// recall of missing pages, host pool -> page-cache slots, for up to GATHER_MAX_LAYERS layers in one launch;
// heads: FKV_HEADS_* (all, flagged only, unflagged only -- by each layer's own flags)
constexpr int GATHER_MAX_LAYERS = 8;
struct GatherLayers {
  int n;
  PoolDesc pd[GATHER_MAX_LAYERS];
  const uint16_t* host_pool[GATHER_MAX_LAYERS];
  const int32_t* miss[GATHER_MAX_LAYERS];
  const uint8_t* flags[GATHER_MAX_LAYERS];
};
void launch_gather(const Dims& d, const GatherLayers& gl, int heads, hipStream_t st);
// returns the number of splits written per KV head
int  launch_attn(const Dims& d, const PoolDesc& pd, const uint16_t* q, const int32_t* act_ids,
                 const int32_t* new_ids, const int32_t* act_slots, const int32_t* new_slots,
                 const uint8_t* flags, int use, float* part_o, float* part_ml, int max_splits,
                 int* counters, float* out, Geom g, hipStream_t st, hipEvent_t ev_begin, hipEvent_t ev_end,
                 long long* tstamp);
void launch_fill_zero(int* p, int n, hipStream_t st);       // p[0..n) = 0, by a kernel
void launch_read_page(const uint16_t* unit, uint16_t* out_token_major, hipStream_t st);
void launch_export_nhd(const Dims& d, const PoolDesc& pd, const int32_t* act_ids, const int32_t* new_ids,
                       const int32_t* act_slots, const int32_t* new_slots, const uint8_t* flags, int use,
                       uint16_t* out, int32_t* slot_pages, int n_slots, Geom g, hipStream_t st,
                       const int32_t* skip_missing = nullptr);   // miss lists: leave the pages they name to the streamed recall
// recall of the missing pages into their page-cache slots AND, converted, into an NHD pool
void launch_gather_nhd(const Dims& d, const PoolDesc& pd, const uint16_t* host_pool, const int32_t* miss,
                       const uint8_t* flags, int heads, uint16_t* nhd, int n_slots, int n_sink, hipStream_t st);

}  // namespace fkv
