// Device code of the "step" roles: token append + incremental summaries, correction test, page weights,
// and (by the last scoring block of each KV head) softmax -> group-mean pooling -> top-k.
// One launch; blocks take roles by index, because the three jobs do not depend on each
// other inside a step: the page being appended to is never a candidate, and a page that
// becomes a candidate had its summary completed at least a window ago.
//
// The selected page ids must be reproducible bit for bit, so the arithmetic that
// decides them is restricted to IEEE fp32/fp64 operations in a fixed order
// (this file is compiled with -ffp-contract=off; FMAs are written explicitly
// and only where the product is exact, so fusing cannot change the result):
//   weight:  128 exact products summed as 16 chunks of 8 consecutive channels,
//            left to right, then an adjacent-pair tree over the 16 chunk sums
//            (the xor-1,2,4,8 butterfly of a 16-lane group), times fl32(1/sqrt(128));
//   softmax: x = P - max; t = x * fl32(log2 e); n = rint(t); f = t - n;
//            degree-6 Horner in f with separate multiply and add; ldexp(., n);
//            0 below t < -64; E = rint(e * 2^31) as integer; Z = integer sum of E;
//   pooling: fl32( (sum_g fp64(E_g) / fp64(Z_g), g ascending) / fp64(G) ); the quotients are the
//            correctly rounded ones, computed from a reciprocal of Z_g with fused multiply-add
//            corrections (see div_rn);
//            (alternatives, App. B.2: fl32(max_g E_g / Z_g); the fp32 sum of the weights in head
//            order divided by G, or their maximum; the weight of the group's mean or maximum query)
//   top-k:   radix select on the order-preserving image of the fp32 bit pattern, ties to the
//            lower page id.
#pragma once
#include "fkv_device.h"
#include "fkv_plan_dev.h"

#pragma clang fp contract(off)

namespace fkv {

#define FKV_STAMP(a, head, i) do { if ((a).tstamp && (head) == 0 && threadIdx.x == 0) (a).tstamp[i] = wall_clock64(); } while (0)

#ifndef FKV_STEP_THREADS
#define FKV_STEP_THREADS 512
#endif
#ifndef FKV_SCORE_PASSES
#define FKV_SCORE_PASSES 4
#endif
constexpr int STEP_THREADS = FKV_STEP_THREADS;         // >= 256 (the radix histograms have 256 bins)
constexpr int STEP_WAVES = STEP_THREADS / 64;
constexpr int SCORE_PASSES = FKV_SCORE_PASSES;         // most passes a scoring block can make (StepArgs::passes <= this)
constexpr int PAGES_PER_PASS = STEP_WAVES * 4;         // a wave scores 4 pages per pass

struct StepArgs {
  int roles;                 // ROLE_* bits
  int batch, n_q, n_kv, k, max_pages;
  Geom g;                    // geometry with the appended token counted
  // append
  PoolDesc pd;
  uint16_t* summ;
  const uint16_t* k_new;
  const uint16_t* v_new;
  // correction test
  const uint16_t* q;
  const uint16_t* q_prev;
  uint16_t* q_stage;
  int have_prev;
  float tau;
  int corr_pool;             // FKV_CORR_*
  uint8_t* flags;
  uint8_t* flags_user;
  double* cosine;
  // selection
  int sel_pool;              // FKV_POOL_*
  float* P;
  float* score;
  int32_t* ids;
  int32_t* ids_user;
  int* counters;
  int blocks_per_head;       // scoring blocks of a KV head; block i takes chunks i, i + blocks_per_head, ...
  int passes;                // passes of PAGES_PER_PASS pages a scoring block makes (1 .. SCORE_PASSES)
  int staged;                // the G x n_cand weights fit in LDS next to the keys
  int fuse_select;           // the last scoring block of a head runs its selection (else: a second launch does)
  int select_only;           // this launch: one block per head, selection only
  float* bmax;               // if not null: [heads][bmax_stride][MAX_G], every scoring block leaves the per-head maxima of
  int bmax_stride;           // the weights it wrote (for a selection spread over several blocks per head)
  long long* tstamp;         // debug: 100 MHz timestamps of head 0's phases (may be null)
  unsigned long long* tagged; // if not null: [heads][k], every picked id once more as (epoch << 32 | id): a block of
  int epoch;                  // this launch that waits for the selection polls the word it needs
  // KV in a host pool: the selecting block also makes the head's recall plan (fkv_plan_dev.h).  plan_new_slots null:
  // not here.  The tagged words then carry, instead of the bare id, what a waiting attention wave needs to fetch the
  // page: tagged_pick() of (page id, slot, miss).
  const int32_t* plan_act_ids;
  const int32_t* plan_act_slots;
  int32_t* plan_new_slots;
  int32_t* plan_miss;
  int plan_lds_off;           // where the plan's LDS starts, in 32-bit words of the block's dynamic LDS
};


// ---------------------------------------------------------------------------------
// role: append one token (Sec. 3.2 summaries; Sec. 4.2 paged layout).  128 active threads.
// ---------------------------------------------------------------------------------
template <int DT>
__device__ __forceinline__ void append_role(const StepArgs& a, int head) {
  const int c = threadIdx.x;
  if (c >= D) return;   // 128 of the block's threads
  const int b = head / a.n_kv, m = head % a.n_kv;
  const int pos = a.g.L - 1, page = pos / PG, t = pos % PG;
  const uint16_t kb = a.k_new[(size_t)head * D + c];
  const uint16_t vb = a.v_new[(size_t)head * D + c];
  uint16_t* pmax = a.summ + summ_idx(b, m, a.n_kv, 0, a.max_pages, page) + c;
  uint16_t* pmin = a.summ + summ_idx(b, m, a.n_kv, 1, a.max_pages, page) + c;
  uint16_t omax = kb, omin = kb;
  if (t != 0) { omax = *pmax; omin = *pmin; }
  uint16_t* unit = a.pd.pool + (head_base(a.pd, b, m, a.n_kv) + resident_unit(a.pd, page)) * UNIT_ELEMS;
  unit[k_elem_off(t, c)] = kb;
  unit[v_elem_off(t, c)] = vb;
  const float kf = Unpack<DT>::one(kb);
  if (t == 0 || kf > Unpack<DT>::one(omax)) *pmax = kb;
  if (t == 0 || kf < Unpack<DT>::one(omin)) *pmin = kb;
}

// ---------------------------------------------------------------------------------
// role: correction test (Sec. 3.1, 3.3).  One wave per query head, fp64.
// ---------------------------------------------------------------------------------
template <int DT, int G, int WAVES = STEP_WAVES>
__device__ __forceinline__ void corr_role(const StepArgs& a, int head) {
  __shared__ double cg[MAX_G];
  const int b = head / a.n_kv, m = head % a.n_kv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int gg = wave; gg < G; gg += WAVES) {
    const size_t off = (size_t)(b * a.n_q + m * G + gg) * D;
    double cosv = 0.0;
    uint32_t qw;
    if (a.have_prev) cosv = head_cosine<DT>(a.q + off, a.q_prev + off, lane, &qw);
    else qw = *reinterpret_cast<const uint32_t*>(a.q + off + lane * 2);
    *reinterpret_cast<uint32_t*>(a.q_stage + off + lane * 2) = qw;
    if (lane == 0) {
      cg[gg] = cosv;
      a.cosine[b * a.n_q + m * G + gg] = cosv;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    uint8_t f = 1;
    if (a.have_prev) f = (uint8_t)pooled_flag(cg, G, a.tau, a.corr_pool);
    a.flags[head] = f;
    if (a.flags_user) a.flags_user[head] = f;
  }
}

// Scores can be negative in the variants that pool the weights themselves: map the fp32 bit
// pattern to an unsigned key with the same order (-0 counts as +0), and back.
__device__ __forceinline__ uint32_t score_key(float sc) {
  const uint32_t u = __float_as_uint(sc + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_score(uint32_t key) {
  return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

// ---------------------------------------------------------------------------------
// role: page weights P^h_j from the min-max summaries (Sec. 3.2).
// A 16-lane group owns one page: lane c8 holds channels 8*c8 .. 8*c8+7 of kmax and
// kmin (one 16-byte load each, 1 KiB contiguous per wave and array), so a wave
// scores 4 pages and a block 16 pages.
// ---------------------------------------------------------------------------------
template <int DT, int G, bool QMODE, int WAVES = STEP_WAVES>
__device__ __forceinline__ void score_pages(const StepArgs& a, int head, int chunk) {
  constexpr int PAGES_PER_PASS = WAVES * 4;               // (of this block size)
  const int b = head / a.n_kv, m = head % a.n_kv;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = lane >> 4, c8 = lane & 15;
  const int pages_per_chunk = PAGES_PER_PASS * a.passes;
  if (chunk * pages_per_chunk >= a.g.n_cand) return;      // a block that only exists to run the selection
  // all summary loads of a chunk's passes first, then q: everything is in flight at once
  uint4 wmax[SCORE_PASSES], wmin[SCORE_PASSES];
  int page[SCORE_PASSES];
  auto load_chunk = [&](int ch) {
#pragma unroll
    for (int ps = 0; ps < SCORE_PASSES; ++ps) {
      const int j = ch * pages_per_chunk + ps * PAGES_PER_PASS + wave * 4 + grp;
      page[ps] = (ps < a.passes && j < a.g.n_cand) ? a.g.cand_lo + j : -1;
      const int pg = a.g.cand_lo + (j < a.g.n_cand ? j : 0);
      if (ps < a.passes) {
        wmax[ps] = *reinterpret_cast<const uint4*>(a.summ + summ_idx(b, m, a.n_kv, 0, a.max_pages, pg) + c8 * 8);
        wmin[ps] = *reinterpret_cast<const uint4*>(a.summ + summ_idx(b, m, a.n_kv, 1, a.max_pages, pg) + c8 * 8);
      }
    }
  };
  load_chunk(chunk);
  float f[G][8];
#pragma unroll
  for (int gg = 0; gg < G; ++gg) {
    const uint4 wq = *reinterpret_cast<const uint4*>(a.q + (size_t)(b * a.n_q + m * G + gg) * D + c8 * 8);
    unpack8<DT>(wq, f[gg]);
  }
  // Variants that pool the QUERY over the group (App. B.2, MeanQ / MaxQ): one pooled query per KV
  // head takes the place of head 0 of the group, and only its row of P is written.
  constexpr int NG = QMODE ? 1 : G;                       // rows of P this launch writes per KV head
  if (QMODE) {
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      float acc = f[0][c];
#pragma unroll
      for (int gg = 1; gg < G; ++gg) acc = a.sel_pool == 4 ? acc + f[gg][c] : fmaxf(acc, f[gg][c]);
      // fp32 quotient by way of fp64: correctly rounded (53 >= 2 * 24 + 2 bits)
      if (a.sel_pool == 4) acc = (float)((double)acc / (double)G);
      f[0][c] = acc;
    }
  }
  const float scale = 0x1.6a09e6p-4f;   // fl32(1/sqrt(128))
  float* const prow = a.P + (size_t)(b * a.n_q + m * G + (c8 < NG ? c8 : 0)) * a.max_pages;
  float best = -__builtin_inff();                         // largest weight this lane has written (query head c8)
  // a block of a big scan takes every blocks_per_head-th chunk of its head, one after the other
  for (int ch = chunk; ch * pages_per_chunk < a.g.n_cand; ch += a.blocks_per_head) {
  if (ch != chunk) load_chunk(ch);
#pragma unroll
  for (int ps = 0; ps < SCORE_PASSES; ++ps) {
    if (ps >= a.passes) break;
    float kx[8], kn[8];
    unpack8<DT>(wmax[ps], kx);
    unpack8<DT>(wmin[ps], kn);
    float mine = 0.0f;                                    // the total of query head c8, for lanes c8 < NG
#pragma unroll
    for (int gg = 0; gg < NG; ++gg) {
      // chunk sum, left to right.  The product q_c * (q_c >= 0 ? kmax_c : kmin_c) of two 16-bit
      // floats is exact in fp32, so the fma rounds once, exactly like "s + product"; a mean
      // query is a full fp32 number, so there the product is rounded on its own first.
      float s;
      if (QMODE) {
        s = f[0][0] * (f[0][0] >= 0.0f ? kx[0] : kn[0]);
#pragma unroll
        for (int c = 1; c < 8; ++c) {
          const float pr = f[0][c] * (f[0][c] >= 0.0f ? kx[c] : kn[c]);
          s = s + pr;
        }
      } else {
        s = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) s = __builtin_fmaf(f[gg][c], f[gg][c] >= 0.0f ? kx[c] : kn[c], s);
      }
      // adjacent-pair tree over the 16 chunk sums (xor 1, 2 in quads; the mirrors pair lanes
      // that hold equal partial sums' complements, which is the same tree); every lane ends up
      // with the total
      s = s + __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(s), 0xB1, 0xf, 0xf, false));
      s = s + __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(s), 0x4E, 0xf, 0xf, false));
      s = s + __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(s), 0x141, 0xf, 0xf, false));
      s = s + __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(s), 0x140, 0xf, 0xf, false));
      mine = c8 == gg ? s : mine;
    }
    // one store per pass: lane c8 of a page's 16 lanes writes the weight of query head c8
    // (device-scope only if a block of this launch is going to read it)
    if (c8 < NG && page[ps] >= 0) {
      if (a.fuse_select) st_dev(prow + page[ps], mine * scale);
      else prow[page[ps]] = mine * scale;
      best = fmaxf(best, mine * scale);
    }
  }
  }
  if (a.bmax) {
    // the block's per-head maxima, for whoever needs the head's: over the wave's four 16-lane groups, then
    // over the waves through LDS; plain stores (the readers are later launches)
    __shared__ float s_best[WAVES][MAX_G];
    best = fmaxf(best, __shfl_xor(best, 16, 64));
    best = fmaxf(best, __shfl_xor(best, 32, 64));
    if (lane < NG) s_best[wave][lane] = best;
    __syncthreads();
    if (threadIdx.x < NG) {
      float v = s_best[0][threadIdx.x];
#pragma unroll
      for (int w = 1; w < WAVES; ++w) v = fmaxf(v, s_best[w][threadIdx.x]);
      a.bmax[((size_t)head * a.bmax_stride + chunk) * MAX_G + threadIdx.x] = v;
    }
  }
}

template <int DT, int G, int WAVES = STEP_WAVES>
__device__ __forceinline__ void score_role(const StepArgs& a, int head, int chunk) {
  if (a.sel_pool >= 4) score_pages<DT, G, true, WAVES>(a, head, chunk);
  else                 score_pages<DT, G, false, WAVES>(a, head, chunk);
}

// ---------------------------------------------------------------------------------
// softmax -> group mean -> top-k for one KV head, by one 256-thread block.
// ---------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t softmax_fixed(float p, float mx) {
  const float x = p - mx;
  const float t = x * 0x1.715476p+0f;          // fl32(log2 e)
  const float n = __builtin_rintf(t);
  const float f = t - n;
  float r = 0x1.430912p-13f;
  r = r * f; r = r + 0x1.5d87fep-10f;
  r = r * f; r = r + 0x1.3b2ab6p-7f;
  r = r * f; r = r + 0x1.c6b08ep-5f;
  r = r * f; r = r + 0x1.ebfbep-3f;
  r = r * f; r = r + 0x1.62e43p-1f;
  r = r * f; r = r + 1.0f;
  // e = ldexp(r, n) is exact here (n >= -64), and so is e * 2^31: one ldexp gives the same number
  float e31 = __builtin_ldexpf(r, (int)n + 31);
  if (t < -64.0f) e31 = 0.0f;
  return (uint32_t)__builtin_rintf(e31);
}

// A reciprocal of b good to an ulp or two: the hardware's approximation (a dozen bits would do)
// sharpened by three Newton steps.
__device__ __forceinline__ double reciprocal_near(double b) {
  double y = __builtin_amdgcn_rcp(b);
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const double e = __builtin_fma(-b, y, 1.0);
    y = __builtin_fma(y, e, y);
  }
  return y;
}

// The correctly rounded fp64 quotient a / b of integers 0 <= a <= b < 2^48 from such a y (one
// reciprocal per head, not one division per candidate): q = a * y corrected twice with the exact
// remainder r = a - b * q.  After the first correction q is within an ulp; the second leaves an
// error of at most |r| * |y - 1/b| <= 2^-52 ulp, and a / b with b < 2^48 is either representable or at
// least 2^-49 ulp away from the nearest rounding boundary, so the rounding cannot go wrong.
__device__ __forceinline__ double div_rn(double a, double b, double y) {
  double q = a * y;
  double r = __builtin_fma(-b, q, a);
  q = __builtin_fma(r, y, q);
  r = __builtin_fma(-b, q, a);
  return __builtin_fma(r, y, q);
}

// pooled score of one candidate from the G per-head values e[] (softmax numerators, or the bits of
// the weights themselves), mode = FKV_POOL_*; zd = the heads' integer sums Z, zr = RN(1 / Z)
template <int G>
__device__ __forceinline__ float pooled_score(const uint32_t* e, const double* zd, const double* zr, int mode) {
  if (mode <= 1) {
    // mean (the method) or maximum over the group of the softmax values, in fp64
    double acc = div_rn((double)e[0], zd[0], zr[0]);
#pragma unroll
    for (int gg = 1; gg < G; ++gg) {
      const double sg = div_rn((double)e[gg], zd[gg], zr[gg]);
      if (mode == 0) acc = acc + sg;
      else acc = sg > acc ? sg : acc;
    }
    return mode == 0 ? (float)(acc / (double)G) : (float)acc;
  }
  // mean or maximum of the weights themselves in fp32, head order; or the pooled query's weight
  float acc = __uint_as_float(e[0]);
#pragma unroll
  for (int gg = 1; gg < G; ++gg) {
    if (mode == 2) acc = acc + __uint_as_float(e[gg]);
    else if (mode == 3) acc = fmaxf(acc, __uint_as_float(e[gg]));
  }
  return mode == 2 ? (float)((double)acc / (double)G) : acc;
}

// ---------------------------------------------------------------------------------
// Block-wide top-kk of n keys held in LDS, ties to the lower index: emit(pos, j) is called for the
// chosen j in ascending order of j with pos = 0 .. kk-1 (whichever thread owns j calls it).
// Before the call (and a barrier): hist[3] holds the counts of the keys' top bytes, hist[0..2] zeros.
// 1 <= kk <= n.
// ---------------------------------------------------------------------------------
template <typename Emit>
__device__ __forceinline__ void radix_topk(const uint32_t* key, int n, int kk, uint32_t (*hist)[256], uint32_t* s_scan,
                                           Emit emit) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // radix select: the kk-th largest key, one byte at a time from the top.  Every wave scans
  // the histogram itself (lane l owns bins 255-4l .. 252-4l), so a pass costs one barrier.
  // It ends early once every key of the chosen bin is wanted: then "all keys from that bin
  // upwards" is the answer and the lower bytes need not be resolved (every wave sees the same
  // histogram, so the whole block takes the exit together).
  uint32_t prefix = 0, remaining = (uint32_t)kk;
  uint32_t T = 0, take_eq = 0;                       // take keys > T, and the first take_eq keys == T
  bool resolved = false;
#pragma unroll
  for (int pass = 3; pass >= 0; --pass) {
    if (resolved) continue;
    const int shift = pass * 8;
    if (pass != 3) {
      for (int j = tid; j < n; j += STEP_THREADS) {
        const uint32_t kj = key[j];
        if ((kj >> (shift + 8)) == prefix) atomicAdd(&hist[pass][(kj >> shift) & 255u], 1u);
      }
      __syncthreads();
    }
    uint32_t c[4], tot = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) { c[i] = hist[pass][255 - 4 * lane - i]; tot += c[i]; }
    const uint32_t incl = wave_scan_u32(tot);
    uint32_t above = incl - tot;                     // keys in bins above this lane's
    const bool mine = above < remaining && remaining <= incl;   // exactly one lane
    uint32_t need = remaining - above;
    int found = 0;
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      if (found == i && c[i] < need) { need -= c[i]; found = i + 1; }
    }
    const unsigned long long pick = __ballot(mine);
    const int src = __builtin_ctzll(pick);
    const uint32_t cf = found == 0 ? c[0] : found == 1 ? c[1] : found == 2 ? c[2] : c[3];
    remaining = (uint32_t)__builtin_amdgcn_readlane((int)need, src);          // how many to take inside the bin
    const uint32_t in_bin = (uint32_t)__builtin_amdgcn_readlane((int)cf, src); // how many it holds
    const uint32_t bin = (uint32_t)__builtin_amdgcn_readlane(255 - 4 * lane - found, src);
    prefix = (prefix << 8) | bin;
    if (pass == 0) {
      T = prefix;                                    // the kk-th largest key itself;
      take_eq = remaining;                           // of the keys equal to it, the lowest ids
      resolved = true;
    } else if (remaining == in_bin && (prefix << shift) != 0) {
      T = (prefix << shift) - 1;                     // everything from the bin's lowest key upwards
      take_eq = 0;
      resolved = true;
    }
  }

  // ordered compaction: thread t owns the contiguous ids [t*per, (t+1)*per)
  const int per = (n + STEP_THREADS - 1) / STEP_THREADS;
  const int j0 = tid * per, j1 = min(n, j0 + per);
  uint32_t cnt = 0;                                  // low 16 bits: keys > T, high 16 bits: keys == T
  for (int j = j0; j < j1; ++j) {
    const uint32_t kj = key[j];
    cnt += (kj > T ? 1u : 0u) + (kj == T ? 0x10000u : 0u);
  }
  const uint32_t incl = wave_scan_u32(cnt);
  if (lane == 63) s_scan[wave] = incl;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += s_scan[w];
  const uint32_t excl = base + incl - cnt;
  uint32_t gt_before = excl & 0xffffu, eq_before = excl >> 16;
  for (int j = j0; j < j1; ++j) {
    const uint32_t kj = key[j];
    if (kj > T || (kj == T && eq_before < take_eq)) {
      const uint32_t pos = gt_before + min(eq_before, take_eq);
      emit((int)pos, j);
    }
    gt_before += (kj > T);
    eq_before += (kj == T);
  }
}

// Most candidates of a KV head the selection keeps in registers (G values each).  The layer kernel
// has the registers for 4 per thread anyway (its attention part needs more); the step kernel alone
// would lose occupancy of its scoring blocks above 2 per thread when G > 4.
__host__ __device__ constexpr int regs_candidates(int G, bool roomy) { return ((roomy || G <= 4) ? 4 : 2) * STEP_THREADS; }

template <int U> struct UnrollBy { static constexpr int value = U; };

// phase marks of the selection, kept in registers until its end (investigation builds only)
#ifdef FKV_SEL_STAMPS
#define FKV_SEL_MARK(i) sel_t##i = wall_clock64()
#else
#define FKV_SEL_MARK(i)
#endif

// a page weight: written earlier in this very launch by another block (device-scope read), or by a
// launch that has ended (plain read)
__device__ __forceinline__ float ld_weight(const float* p, bool same_launch) {
  return same_launch ? ld_dev(p) : *p;
}

template <int G, bool STAGED, bool ROOMY>
__device__ __forceinline__ void select_block(const StepArgs& a, int head, uint32_t* key) {
  __shared__ float s_redf[STEP_WAVES][G];
  __shared__ unsigned long long s_redz[STEP_WAVES][G];
  __shared__ uint32_t hist[4][256];
  __shared__ uint32_t s_scan[STEP_WAVES];

  const int b = head / a.n_kv, m = head % a.n_kv, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n = a.g.n_cand, lo = a.g.cand_lo, kk = a.g.k_eff, k = a.k;
  int32_t* out = a.ids + (size_t)head * k;
  int32_t* outu = a.ids_user ? a.ids_user + (size_t)head * k : nullptr;
  // No global store is issued before the last barrier of this function: a barrier waits for
  // the acknowledgement of every store the wave has in flight, a full trip to memory.
  // a picked id goes out three ways: the layer's id list, the caller's copy, and (one-launch layer-step) tagged
  // with the step's epoch in one 64-bit word, so that a waiting attention wave sees "this step's id" in one read
  unsigned long long* tag = a.tagged ? a.tagged + (size_t)head * k : nullptr;
  const unsigned long long tag_hi = (unsigned long long)(uint32_t)a.epoch << 32;
  // With a recall plan to make, the ids are only collected in the plan's LDS here and everything goes out after it.
  int32_t* plan_sm = reinterpret_cast<int32_t*>(key) + a.plan_lds_off;
  int32_t* plan_nid = a.plan_new_slots ? plan_sm + 4 * k : nullptr;
  auto put_id = [&](int pos, int id) {
    if (plan_nid) { plan_nid[pos] = id; return; }
    __hip_atomic_store(out + pos, id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tag) __hip_atomic_store(tag + pos, tag_hi | (uint32_t)id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (outu) outu[pos] = id;
  };
  auto plan_and_publish = [&]() {
    if (!plan_nid) return;
    __syncthreads();                                   // the ids are all in LDS
    plan_head<STEP_THREADS>(out, a.plan_act_ids + (size_t)head * k, a.plan_act_slots + (size_t)head * k,
                            a.plan_new_slots + (size_t)head * k, a.plan_miss + (size_t)head * (1 + 3 * k), k, a.g.n_full,
                            plan_sm, true);
    const int32_t* nslot = plan_sm + 5 * k;
    for (int i = tid; i < k; i += STEP_THREADS) {
      const int id = plan_nid[i], s = nslot[i];
      __hip_atomic_store(out + i, id, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (tag) __hip_atomic_store(tag + i, tag_hi | tagged_pick(id, s & (TAGGED_MAX_SLOTS - 1), (s & PLAN_MISS_BIT) != 0),
                                  __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (outu) outu[i] = id;
    }
  };
  if (kk == 0) {
    for (int i = tid; i < k; i += STEP_THREADS) put_id(i, -1);
    plan_and_publish();
    return;
  }
#ifdef FKV_SEL_STAMPS
  long long sel_t0 = 0, sel_t1 = 0, sel_t2 = 0, sel_t3 = 0, sel_t4 = 0;
#endif
  FKV_SEL_MARK(0);
  const float* Pm = a.P + (size_t)(b * a.n_q + m * G) * a.max_pages + lo;
  uint32_t* pw = key + n;                              // [G][n]: weights, later their fixed-point softmax
  constexpr bool staged = STAGED;                      // else: re-read the weights from memory in each pass
  const bool same_launch = a.select_only == 0;         // the weights come from scoring blocks of this launch
  const int mode = a.sel_pool;                         // FKV_POOL_*
  const bool soft = mode <= 1;                         // the variants that pool softmax values
  const int ng = mode >= 4 ? 1 : G;                    // rows of P in use (pooled query: the group's first)
#pragma unroll
  for (int p = 0; p < 4; ++p)
    if (tid < 256) hist[p][tid] = 0;

  // A few candidates per thread stay in registers from the load to the key: no staging in LDS.
  const bool in_regs = n <= regs_candidates(G, ROOMY);
  auto front_in_regs = [&](auto uc) {
    constexpr int U = decltype(uc)::value;
    uint32_t e[U][G];                                  // bits of the weights, then softmax numerators
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = min(tid + u * STEP_THREADS, n - 1);
#pragma unroll
      for (int gg = 0; gg < G; ++gg)
        e[u][gg] = gg < ng ? __float_as_uint(ld_weight(Pm + (size_t)gg * a.max_pages + j, same_launch)) : 0u;
    }
    double zd[G];
#pragma unroll
    for (int gg = 0; gg < G; ++gg) zd[gg] = 1.0;
    if (soft) {
      float mx[G];
#pragma unroll
      for (int gg = 0; gg < G; ++gg) mx[gg] = -__builtin_inff();
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (tid + u * STEP_THREADS < n) {
#pragma unroll
          for (int gg = 0; gg < G; ++gg) mx[gg] = fmaxf(mx[gg], __uint_as_float(e[u][gg]));
        }
#pragma unroll
      for (int gg = 0; gg < G; ++gg) {
        const float w = wave_max_f32(mx[gg]);
        if (lane == 0) s_redf[wave][gg] = w;
      }
      __syncthreads();
#pragma unroll
      for (int gg = 0; gg < G; ++gg) {
        float v = s_redf[0][gg];
#pragma unroll
        for (int w = 1; w < STEP_WAVES; ++w) v = fmaxf(v, s_redf[w][gg]);
        mx[gg] = v;
      }
      FKV_SEL_MARK(1);
      unsigned long long z[G];
#pragma unroll
      for (int gg = 0; gg < G; ++gg) z[gg] = 0;
#pragma unroll
      for (int u = 0; u < U; ++u) {
#pragma unroll
        for (int gg = 0; gg < G; ++gg) {
          e[u][gg] = softmax_fixed(__uint_as_float(e[u][gg]), mx[gg]);
          if (tid + u * STEP_THREADS < n) z[gg] += e[u][gg];
        }
      }
#pragma unroll
      for (int gg = 0; gg < G; ++gg) {
        const unsigned long long w = wave_sum_u48(z[gg]);
        if (lane == 0) s_redz[wave][gg] = w;
      }
      __syncthreads();
#pragma unroll
      for (int gg = 0; gg < G; ++gg) {
        unsigned long long v = 0;
#pragma unroll
        for (int w = 0; w < STEP_WAVES; ++w) v += s_redz[w][gg];
        zd[gg] = (double)v;
      }
    } else {
      FKV_SEL_MARK(1);
    }
    double zr[G];
#pragma unroll
    for (int gg = 0; gg < G; ++gg) zr[gg] = reciprocal_near(zd[gg]);
    FKV_SEL_MARK(2);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = tid + u * STEP_THREADS;
      const uint32_t kj = score_key(pooled_score<G>(e[u], zd, zr, mode));
      if (j < n) {
        key[j] = kj;
        atomicAdd(&hist[3][kj >> 24], 1u);
      }
    }
  };
  if (in_regs) {
    if (!soft) __syncthreads();                        // the histograms are clear (else: barriers below)
    if (n <= STEP_THREADS) front_in_regs(UnrollBy<1>{});
    else if (n <= 2 * STEP_THREADS) front_in_regs(UnrollBy<2>{});
    else if constexpr (regs_candidates(G, ROOMY) > 2 * STEP_THREADS) front_in_regs(UnrollBy<4>{});
  } else {
  // stage the weights of this head's G query heads in LDS (one device-scope read each, 8 x G
  // of them in flight per thread) and take the per-head maximum over the candidates
  float mx[G];
#pragma unroll
  for (int gg = 0; gg < G; ++gg) mx[gg] = -__builtin_inff();
  // Each loop over the candidates handles U of them per thread and trip, all loads first, so
  // that U x G independent chains are in flight; U is matched to n, because a trip works on
  // U x STEP_THREADS candidates whether they exist or not.
  auto stage_and_max = [&](auto uc) {
    constexpr int U = decltype(uc)::value;
    for (int j0 = tid; j0 < n; j0 += U * STEP_THREADS) {
      float v[U][G];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = min(j0 + u * STEP_THREADS, n - 1);
#pragma unroll
        for (int gg = 0; gg < G; ++gg) v[u][gg] = gg < ng ? ld_weight(Pm + (size_t)gg * a.max_pages + j, same_launch) : 0.0f;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = j0 + u * STEP_THREADS;
        if (j < n) {
#pragma unroll
          for (int gg = 0; gg < G; ++gg) {
            if (staged) pw[gg * n + j] = __float_as_uint(v[u][gg]);
            mx[gg] = fmaxf(mx[gg], v[u][gg]);
          }
        }
      }
    }
  };
  if (soft || staged) {
    if (n <= 2 * STEP_THREADS) stage_and_max(UnrollBy<2>{});
    else if (n <= 4 * STEP_THREADS) stage_and_max(UnrollBy<4>{});
    else stage_and_max(UnrollBy<8>{});
  }
#pragma unroll
  for (int gg = 0; gg < G; ++gg) {
    const float w = wave_max_f32(mx[gg]);
    if (lane == 0) s_redf[wave][gg] = w;
  }
  __syncthreads();
#pragma unroll
  for (int gg = 0; gg < G; ++gg) {
    float v = s_redf[0][gg];
#pragma unroll
    for (int w = 1; w < STEP_WAVES; ++w) v = fmaxf(v, s_redf[w][gg]);
    mx[gg] = v;
  }
  FKV_SEL_MARK(1);
  // fixed-point softmax numerators in place, integer denominators (a sum of integers: no order to fix)
  unsigned long long z[G];
#pragma unroll
  for (int gg = 0; gg < G; ++gg) z[gg] = 0;
  auto numerators = [&](auto uc) {
    constexpr int U = decltype(uc)::value;
    for (int j0 = tid; j0 < n; j0 += U * STEP_THREADS) {
      float v[U][G];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = min(j0 + u * STEP_THREADS, n - 1);
#pragma unroll
        for (int gg = 0; gg < G; ++gg)
          v[u][gg] = staged ? __uint_as_float(pw[gg * n + j]) : ld_weight(Pm + (size_t)gg * a.max_pages + j, same_launch);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int j = j0 + u * STEP_THREADS;
#pragma unroll
        for (int gg = 0; gg < G; ++gg) {
          const uint32_t e = softmax_fixed(v[u][gg], mx[gg]);
          if (j < n) {
            if (staged) pw[gg * n + j] = e;
            z[gg] += e;
          }
        }
      }
    }
  };
  if (soft) {
    if (n <= 2 * STEP_THREADS) numerators(UnrollBy<2>{});
    else numerators(UnrollBy<4>{});
  }
#pragma unroll
  for (int gg = 0; gg < G; ++gg) {
    const unsigned long long w = wave_sum_u48(z[gg]);   // z < 2^31 * ceil(n / threads) < 2^48
    if (lane == 0) s_redz[wave][gg] = w;
  }
  __syncthreads();
  double zd[G];
#pragma unroll
  for (int gg = 0; gg < G; ++gg) {
    unsigned long long v = 0;
#pragma unroll
    for (int w = 0; w < STEP_WAVES; ++w) v += s_redz[w][gg];
    zd[gg] = (double)v;
  }
  double zr[G];
#pragma unroll
  for (int gg = 0; gg < G; ++gg) zr[gg] = reciprocal_near(zd[gg]);
  FKV_SEL_MARK(2);
  // pooled score of each candidate (each thread reads back only what it wrote); the top
  // byte of its key goes straight into the first histogram
  auto pool_and_key = [&](auto uc) {
    constexpr int U = decltype(uc)::value;
  for (int j0 = tid; j0 < n; j0 += U * STEP_THREADS) {
    uint32_t e[U][G];                                // softmax numerators, or the bits of the weights
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = min(j0 + u * STEP_THREADS, n - 1);
#pragma unroll
      for (int gg = 0; gg < G; ++gg) {
        if (staged) e[u][gg] = pw[gg * n + j];
        else if (gg < ng) {
          const float w = ld_weight(Pm + (size_t)gg * a.max_pages + j, same_launch);
          e[u][gg] = soft ? softmax_fixed(w, mx[gg]) : __float_as_uint(w);
        } else e[u][gg] = 0;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int j = j0 + u * STEP_THREADS;
      const float sc = pooled_score<G>(e[u], zd, zr, mode);
      const uint32_t kj = score_key(sc);
      if (j < n) {
        key[j] = kj;
        atomicAdd(&hist[3][kj >> 24], 1u);
      }
    }
  }
  };
  if (n <= 2 * STEP_THREADS) pool_and_key(UnrollBy<2>{});
  else pool_and_key(UnrollBy<4>{});
  }
  __syncthreads();

  FKV_SEL_MARK(3);
  radix_topk(key, n, kk, hist, s_scan, [&](int pos, int j) { put_id(pos, lo + j); });
  FKV_SEL_MARK(4);
  for (int i = kk + tid; i < k; i += STEP_THREADS) put_id(i, -1);   // padding
  plan_and_publish();
#ifdef FKV_SEL_STAMPS
  if (a.tstamp && head == 0 && tid == 0) {
    a.tstamp[40] = sel_t0; a.tstamp[41] = sel_t1; a.tstamp[42] = sel_t2; a.tstamp[43] = sel_t3;
    a.tstamp[44] = sel_t4; a.tstamp[45] = wall_clock64();
  }
#endif
}


// ---------------------------------------------------------------------------------
// role dispatch of one block: bid counts [append blocks][corr blocks][scoring blocks], each
// set present only if its role bit is set; heads = batch * n_kv.
// ---------------------------------------------------------------------------------
template <int DT, int G, bool ROOMY>
__device__ __forceinline__ void step_roles(const StepArgs& a, int bid, uint32_t* dyn_lds) {
  const int heads = a.batch * a.n_kv;
  int head;
  if (a.select_only) {
    head = bid;
  } else {
    if (a.roles & ROLE_APPEND) {
      if (bid < heads) { append_role<DT>(a, bid); return; }
      bid -= heads;
    }
    if (a.roles & ROLE_CORR) {
      if (bid < heads) { corr_role<DT, G>(a, bid); return; }
      bid -= heads;
    }
    head = bid / a.blocks_per_head;
    const int chunk = bid % a.blocks_per_head;
    if (chunk == 0) FKV_STAMP(a, head, 0);
#ifdef FKV_SEL_STAMPS
    if (chunk == 0 && a.tstamp && threadIdx.x == 0) a.tstamp[56 + (head & 7)] = wall_clock64();
#endif
    score_role<DT, G>(a, head, chunk);
    if (chunk == 0) FKV_STAMP(a, head, 1);
    if (!a.fuse_select) return;
    if (a.blocks_per_head == 1) block_release();       // the head's only scoring block: its own weights, once they are out
    else if (!last_block_done(a.counters + head, a.blocks_per_head)) return;
  }
  FKV_STAMP(a, head, 2);
  if (a.staged) select_block<G, true, ROOMY>(a, head, dyn_lds);
  else          select_block<G, false, ROOMY>(a, head, dyn_lds);
  FKV_STAMP(a, head, 8);
#ifdef FKV_SEL_STAMPS
  if (a.tstamp && threadIdx.x == 0) a.tstamp[24 + (head & 7)] = wall_clock64();
#endif
  // the pooled scores, kept for inspection; after the ids, which nothing here should delay
  if (a.g.k_eff > 0)
    for (int j = threadIdx.x; j < a.g.n_cand; j += STEP_THREADS)
      a.score[(size_t)head * a.max_pages + a.g.cand_lo + j] = key_score(dyn_lds[j]);
}

}  // namespace fkv
