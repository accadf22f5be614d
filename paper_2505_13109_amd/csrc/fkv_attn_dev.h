// Device code of sparse decode attention over sink + picked pages + window + open page
// (Sec. 2.1), split over pages with an online softmax; the block that finishes a KV head last
// does the log-sum-exp merge of its splits.
//
// One wavefront owns one 32-token page at a time and keeps everything in registers:
//   S^T[32 tok x 16] = K[32 x 128] . Q^T[128 x 16]       8 x v_mfma_f32_16x16x32
//   O^T[128 x 16]   += V^T[128 x 32 tok] . P^T[32 x 16]   8 (x2: P split hi + lo) MFMAs
// The query group (G <= 8 heads, padded to the 16 columns of the tile) is the N
// dimension of both products, so lane (g = lane % 16, rb = lane / 16) ends the first
// product holding the logits of head g for tokens {rb*4+i, 16+rb*4+i}: exactly the 8
// tokens the same lane must supply as the B operand of the second product (the V page
// is stored in that token order).  Nothing goes through LDS inside the page loop.
#pragma once
#include "fkv_device.h"

namespace fkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

template <int DT> struct Mma;
template <> struct Mma<0> {
  typedef f16x8 vec;
  static __device__ __forceinline__ f32x4 mma(vec a, vec b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
  // p >= 0 split into two storage-type values whose sum carries ~22 bits of p
  static __device__ __forceinline__ void split(const float* p, vec& hi, vec& lo) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const _Float16 h = (_Float16)p[e];
      hi[e] = h;
      lo[e] = (_Float16)(p[e] - (float)h);
    }
  }
};
template <> struct Mma<1> {
  typedef bf16x8 vec;
  static __device__ __forceinline__ f32x4 mma(vec a, vec b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint16_t rne(float x) {
    const uint32_t u = __float_as_uint(x);
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
  }
  static __device__ __forceinline__ void split(const float* p, vec& hi, vec& lo) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint16_t h = rne(p[e]);
      const float hf = __uint_as_float(((uint32_t)h) << 16);
      hi[e] = __builtin_bit_cast(__bf16, h);
      lo[e] = __builtin_bit_cast(__bf16, rne(p[e] - hf));
    }
  }
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr int MAX_MERGE_SPLITS = 256;   // upper bound on splits per KV head

struct AttnArgs {
  PoolDesc pd;
  const uint16_t* q;
  const int32_t* act_ids;    // ACTIVE selection (previous step) and its page-cache slots
  const int32_t* new_ids;    // PENDING selection (this step)
  const int32_t* act_slots;
  const int32_t* new_slots;
  const uint8_t* flags;
  int use;                   // FKV_USE_*: 0 active, 1 pending, 2 by flag
  float* part_o;
  float* part_ml;
  int max_splits, pps, n_splits;
  int* counters;
  float* out;
  Geom g;
  int n_q, n_kv, G, k;
  long long* tstamp;
  // --- when attention shares its launch with the step roles ("fused") ---
  int fused;                 // flags are recomputed here, the new token is taken from k_new/v_new,
                             // a corrected head waits for its selection
  const uint16_t* q_prev;
  int have_prev;
  float tau;
  int corr_pool;
  const uint16_t* k_new;
  const uint16_t* v_new;
  const unsigned long long* tagged;   // [heads][k]: this step's picked ids as (epoch << 32 | id), written by the selection
  int epoch;
  int* status;               // set to 1 if a wait ran out
  // fused, KV in a host pool: the tagged words are tagged_pick() values; a corrected head's wave copies a missing page
  // from the host pool into its slot while it attends over it
  const uint16_t* host_pool; // [heads][max_pages] units
  int max_pages;
};

template <int CH> struct MergeChunk { static constexpr int value = CH; };

// position i of a head's attend list -> HBM unit, page id and number of valid tokens; -1 if empty
struct AttendList {
  const int32_t* ids;
  const int32_t* slots;
  int n_sink, k, n_win, n_full, r;
  bool coherent_ids;         // ids written earlier in this very launch: read them at device scope
};
// have_id: the page id of position i was fetched earlier (`id`), do not load it again
__device__ __forceinline__ int attend_unit(const AttendList& al, const PoolDesc& pd, int i, int& n_valid, int& page,
                                           bool have_id = false, int id_in = -1) {
  n_valid = PG;
  if (i < al.n_sink) { page = i; return i; }
  i -= al.n_sink;
  if (i < al.k) {
    const int id = have_id ? id_in
                 : al.coherent_ids ? __hip_atomic_load(al.ids + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : al.ids[i];
    page = id;
    if (id < 0) return -1;
    return pd.placement == 0 ? id : pd.sel_base + al.slots[i];
  }
  i -= al.k;
  if (i < al.n_win) page = al.n_full - al.n_win + i;
  else { page = al.n_full; n_valid = al.r; }
  if (pd.placement == 0) return page;
  return page < pd.ring_base ? page : pd.ring_base + page % pd.n_ring;
}

// One block of NW wavefronts: attend-list positions [split*pps, (split+1)*pps) of head (b, m),
// wave w takes w, w+NW, ...  `lds` is at least NW*(32 + G*128) floats when NW > 1.
// HOSTFUSED: the variant for a fused launch with the KV in a host pool (a compile-time choice: what it adds to the page
// loop would cost the other launches registers).
template <int DT, int NW, bool HOSTFUSED = false>
__device__ __forceinline__ void attn_block(const AttnArgs& a, int split, int m, int b, float* lds) {
  typedef typename Mma<DT>::vec vec;
  const PoolDesc& pd = a.pd;
  const Geom& g = a.g;
  const int n_q = a.n_q, n_kv = a.n_kv, G = a.G, k = a.k;
  const int head = b * n_kv + m;
#define FKV_ASTAMP(i) do { if (a.tstamp && head == 0 && threadIdx.x == 0) a.tstamp[i] = wall_clock64(); } while (0)
  if (split == 0) FKV_ASTAMP(16);
#ifdef FKV_SEL_STAMPS
  if (split == 0 && a.tstamp && threadIdx.x == 0) a.tstamp[48 + (head & 7)] = wall_clock64();
#endif
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int gq = lane & 15, rb = lane >> 4;
  __shared__ double s_cos[MAX_G];
  __shared__ int s_flag;

  // Q^T operand: lane (g, kb) holds channels (s*4+kb)*8 .. +8 of head g for k-step s
  vec qv[4];
  {
    const uint16_t* qh = a.q + (size_t)(b * n_q + m * G + (gq < G ? gq : 0)) * D;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      uint4 w = *reinterpret_cast<const uint4*>(qh + (s * 4 + rb) * 8);
      if (gq >= G) w = make_uint4(0, 0, 0, 0);
      qv[s] = __builtin_bit_cast(vec, w);
    }
  }

  // In a fused launch the common case is "no correction": fetch the first page id of this wave
  // from the ACTIVE list now, together with the loads of the correction test, instead of after it.
  const int pos0 = split * a.pps + wave;
  const bool spec = a.fused && pos0 >= g.n_sink && pos0 < g.n_sink + k;
  int spec_id = -1;
  if (spec) spec_id = a.act_ids[(size_t)head * k + pos0 - g.n_sink];

  bool pending;
  if (a.fused) {
    // the correction test again, with the arithmetic of the step role, so that this block does
    // not have to wait for that role's result
    if (a.have_prev) {
      for (int gg = wave; gg < G; gg += NW) {
        const size_t off = (size_t)(b * n_q + m * G + gg) * D;
        const double c = head_cosine<DT>(a.q + off, a.q_prev + off, lane, nullptr);
        if (lane == 0) s_cos[gg] = c;
      }
      __syncthreads();
      if (threadIdx.x == 0) s_flag = pooled_flag(s_cos, G, a.tau, a.corr_pool);
      __syncthreads();
      pending = s_flag != 0;
    } else {
      pending = true;
    }
  } else {
    pending = a.use == 1 || (a.use == 2 && a.flags[head] != 0);
  }

  AttendList al;
  al.ids = (pending ? a.new_ids : a.act_ids) + (size_t)head * k;
  al.slots = pd.placement == 0 ? nullptr : (pending ? a.new_slots : a.act_slots) + (size_t)head * k;
  al.n_sink = g.n_sink; al.k = k; al.n_win = g.n_win; al.n_full = g.n_full; al.r = g.r;
  al.coherent_ids = a.fused && pending;
  const int n_att = g.n_sink + k + g.n_win + (g.r > 0 ? 1 : 0);
  const uint16_t* head_pool = pd.pool + (size_t)head * pd.units_per_head * UNIT_ELEMS;
  // the token appended at this step: in a fused launch its K/V may not be in the pool yet
  const int new_page = a.fused ? (g.L - 1) / PG : -1, new_tok = (g.L - 1) % PG;
  const float sl2 = 0.08838834764831845f * 1.4426950408889634f;   // 1/sqrt(d) * log2(e)

  float m_run = -__builtin_inff(), l_run = 0.0f;
  f32x4 acc[8];
#pragma unroll
  for (int cb = 0; cb < 8; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};

  // A corrected head of a fused launch attends with this step's selection, which other blocks of
  // the same launch are still making.  Only the k picked positions of the attend list depend on it:
  // the wave first attends its sink, window and open-page positions (phase 0), then waits for the
  // selection and attends its picked positions (phase 1).  Everything else runs as one phase.
  const bool two_phase = a.fused && pending && k > 0;
  const int pk_lo = g.n_sink, pk_hi = g.n_sink + k;
  const int p_end = min(n_att, (split + 1) * a.pps);
  bool timed_out = false;
  for (int phase = 0; phase < (two_phase ? 2 : 1); ++phase) {
    // first position of this wave, from `from` on, that belongs to the phase and holds a page
    int n_valid = PG, page = -1;
    // a position's page: where in the attend list, which unit of the head's pool, where its bytes are read from, and
    // whether they come from the host pool and have to be put into that unit on the way
    struct Pick { int pos, unit; const uint16_t* src; bool fill; };
    auto find = [&](int from, int& nv, int& pg) -> Pick {
      for (int p2 = from; p2 < p_end; p2 += NW) {
        if (two_phase && ((p2 >= pk_lo && p2 < pk_hi) != (phase == 1))) continue;
        bool have_id = spec && !pending && p2 == pos0;
        int id = spec_id, slot = -1;
        bool miss = false;
        if (two_phase && phase == 1) {
          // Wait for this step's id of the position: the selection writes every picked id as one 64-bit
          // word tagged with the step's epoch.  The block that makes it is one of the scoring blocks of
          // this launch, which all have lower block indices than any attention block and never wait for
          // anything, so it is running or done; the wait is bounded all the same.  The whole wave polls
          // the same word (one request per poll).
          if (timed_out) break;
          const unsigned long long* word = a.tagged + (size_t)head * k + (p2 - pk_lo);
          unsigned long long w2;
          int it = 0;
          while (((w2 = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) >> 32) != (unsigned long long)(uint32_t)a.epoch) {
            if (++it > (1 << 16)) { timed_out = true; break; }   // ~0.1 s
            __builtin_amdgcn_s_sleep(4);
          }
          if (timed_out) {
            if (lane == 0) *a.status = 1;
            break;                                             // the id is not there: read nothing
          }
          have_id = true;
          if constexpr (HOSTFUSED) tagged_unpick((uint32_t)w2, id, slot, miss);
          else id = (int)(uint32_t)w2;
        }
        if (HOSTFUSED && slot >= 0) {
          // KV in a host pool, this step's selection: the slot came with the id (the slot table in memory is being
          // written by another block of this launch); a page the cache does not hold is read from the host pool
          nv = PG;
          pg = id;
          const int u = pd.sel_base + slot;
          const uint16_t* from_pool = head_pool + (size_t)u * UNIT_ELEMS;
          return Pick{p2, u, miss ? a.host_pool + ((size_t)head * a.max_pages + id) * UNIT_ELEMS : from_pool, miss};
        }
        const int u = attend_unit(al, pd, p2, nv, pg, have_id, id);
        if (u >= 0) return Pick{p2, u, head_pool + (size_t)u * UNIT_ELEMS, false};
      }
      return Pick{p_end, -1, nullptr, false};
    };
    // Page loop, software-pipelined: the 16 wave-loads of the next page are issued before the
    // MFMAs of the current one, so a wave that owns several pages keeps 32 KiB in flight.
    const Pick cur = find(pos0, n_valid, page);
    int pos = cur.pos, unit = cur.unit;
    bool fill = cur.fill;
  uint4 kw[8], vw[8];
  if (unit >= 0) {
    const uint4* up = reinterpret_cast<const uint4*>(cur.src) + lane;
#pragma unroll
    for (int j = 0; j < 8; ++j) kw[j] = up[j * 64];
#pragma unroll
    for (int j = 0; j < 8; ++j) vw[j] = up[(8 + j) * 64];
  }
  while (unit >= 0) {
    // next page of this wave, if any
    int nn_valid = PG, npage = -1;
    const Pick nxt = find(pos + NW, nn_valid, npage);
    const int npos = nxt.pos, nunit = nxt.unit;
    uint4 kn[8], vn[8];
    if (nunit >= 0) {
      const uint4* up = reinterpret_cast<const uint4*>(nxt.src) + lane;
#pragma unroll
      for (int j = 0; j < 8; ++j) kn[j] = up[j * 64];
#pragma unroll
      for (int j = 0; j < 8; ++j) vn[j] = up[(8 + j) * 64];
    }
    if (HOSTFUSED && fill) {
      // the page came from the host pool: it goes into its page-cache slot as it is (recall, Sec. 3.3: a corrected
      // head's pages are fetched before it attends; here the wave that attends over the page is the one that fetches it)
      uint4* dp = reinterpret_cast<uint4*>(pd.pool + ((size_t)head * pd.units_per_head + unit) * UNIT_ELEMS) + lane;
#pragma unroll
      for (int j = 0; j < 8; ++j) dp[j * 64] = kw[j];
#pragma unroll
      for (int j = 0; j < 8; ++j) dp[(8 + j) * 64] = vw[j];
    }
    if (page == new_page) {
      // overwrite the new token's key row and value column with the step's inputs
      const uint16_t* kn_h = a.k_new + (size_t)head * D;
      const uint16_t* vn_h = a.v_new + (size_t)head * D;
      const int mb_new = new_tok >> 4;
      if (gq == (new_tok & 15)) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const uint4 w = *reinterpret_cast<const uint4*>(kn_h + (s * 4 + rb) * 8);
          if (mb_new == 0) kw[s * 2] = w; else kw[s * 2 + 1] = w;
        }
      }
      const int kb_new = (new_tok & 15) >> 2, e_new = (new_tok & 3) + 4 * (new_tok >> 4);
      if (rb == kb_new) {
#pragma unroll
        for (int cb = 0; cb < 8; ++cb) {
          const uint32_t v = vn_h[cb * 16 + gq];
          const uint32_t keep = (e_new & 1) ? 0x0000ffffu : 0xffff0000u;
          const uint32_t put = (e_new & 1) ? (v << 16) : v;
          // (no run-time indexing of the register array)
          if ((e_new >> 1) == 0) vw[cb].x = (vw[cb].x & keep) | put;
          if ((e_new >> 1) == 1) vw[cb].y = (vw[cb].y & keep) | put;
          if ((e_new >> 1) == 2) vw[cb].z = (vw[cb].z & keep) | put;
          if ((e_new >> 1) == 3) vw[cb].w = (vw[cb].w & keep) | put;
        }
      }
    }

    f32x4 st[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
        st[mb] = Mma<DT>::mma(__builtin_bit_cast(vec, kw[s * 2 + mb]), qv[s], st[mb]);
    }
    // logits (base 2) of head gq for tokens mb*16 + rb*4 + i
    float sc[8];
    float mx = -__builtin_inff();
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int tok = (e >> 2) * 16 + rb * 4 + (e & 3);
      sc[e] = tok < n_valid ? st[e >> 2][e & 3] * sl2 : -__builtin_inff();
      mx = fmaxf(mx, sc[e]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = fast_exp2(m_run - m_new);
    float p[8], psum = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      p[e] = fast_exp2(sc[e] - m_new);
      psum += p[e];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) acc[cb] *= alpha;
    vec phi, plo;
    Mma<DT>::split(p, phi, plo);
#pragma unroll
    for (int cb = 0; cb < 8; ++cb) {
      const vec va = __builtin_bit_cast(vec, vw[cb]);
      acc[cb] = Mma<DT>::mma(va, phi, acc[cb]);
      acc[cb] = Mma<DT>::mma(va, plo, acc[cb]);
    }
    pos = npos; unit = nunit; n_valid = nn_valid; page = npage; fill = nxt.fill;
    if (nunit >= 0) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { kw[j] = kn[j]; vw[j] = vn[j]; }
    }
  }
  }   // phases
  // A wave whose wait ran out has not read its picked pages: make that visible on the data path.
  // NaN in its sum poisons the block's partial and, through the merge, every output row of the
  // KV head's query group.
  if (timed_out) l_run = __builtin_nanf("");
  if constexpr (HOSTFUSED) {
    // With the KV in a host pool the wave that gives up also leaves the page-cache slot it was to fill unfilled, while
    // the recall plan lists the page as cached: the layer's state cannot be trusted from then on.  Every later step of
    // the layer therefore stays marked -- NaN outputs -- for as long as the flag is up (fkv_health takes it down).
    if (__hip_atomic_load(a.status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) l_run = __builtin_nanf("");
  }
  if (split == 0) FKV_ASTAMP(17);
  // per-wave totals of l over the 4 row blocks
  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);

  float* po = a.part_o + ((size_t)(head * a.max_splits + split) * G) * D;
  float* pml = a.part_ml + ((size_t)(head * a.max_splits + split) * G) * 2;
  if (NW == 1) {
    if (gq < G) {
#pragma unroll
      for (int cb = 0; cb < 8; ++cb) {
        float* dst = po + (size_t)gq * D + cb * 16 + rb * 4;
        st_dev2(dst, acc[cb][0], acc[cb][1]);
        st_dev2(dst + 2, acc[cb][2], acc[cb][3]);
      }
      if (rb == 0) st_dev2(pml + gq * 2, m_run, l_run);
    }
  } else {
    float* sm_m = lds;                    // [NW][16]
    float* sm_l = lds + NW * 16;          // [NW][16]
    float* sm_o = lds + NW * 32;          // [NW][G][D]
    if (rb == 0) sm_m[wave * 16 + gq] = m_run;
    __syncthreads();
    if (split == 0) FKV_ASTAMP(22);
    float M = sm_m[gq];
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, sm_m[w * 16 + gq]);
    // a wave that saw no page has m_run = -inf and zero sums
    const float wgt = (m_run == -__builtin_inff()) ? 0.0f : fast_exp2(m_run - M);
    if (gq < G) {
#pragma unroll
      for (int cb = 0; cb < 8; ++cb)
        *reinterpret_cast<f32x4*>(&sm_o[((size_t)wave * G + gq) * D + cb * 16 + rb * 4]) = acc[cb] * wgt;
      if (rb == 0) sm_l[wave * 16 + gq] = l_run * wgt;
    }
    __syncthreads();
    if (split == 0) FKV_ASTAMP(23);
    if (a.n_splits == 1) {
      // the block has the whole head: normalise and write the output, no partial, no merge
      for (int i = threadIdx.x; i < G * D / 2; i += NW * 64) {
        const int gg = i / (D / 2), c = (i % (D / 2)) * 2;
        float s0 = 0.0f, s1 = 0.0f, den = 0.0f;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          s0 += sm_o[((size_t)w * G + gg) * D + c];
          s1 += sm_o[((size_t)w * G + gg) * D + c + 1];
          den += sm_l[w * 16 + gg];
        }
        const float inv = 1.0f / den;
        *reinterpret_cast<float2*>(a.out + (size_t)(b * n_q + m * G + gg) * D + c) = make_float2(s0 * inv, s1 * inv);
      }
      return;
    }
    for (int i = threadIdx.x; i < G * D / 2; i += NW * 64) {
      const int gg = i / (D / 2), c = (i % (D / 2)) * 2;
      float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        s0 += sm_o[((size_t)w * G + gg) * D + c];
        s1 += sm_o[((size_t)w * G + gg) * D + c + 1];
      }
      st_dev2(po + (size_t)gg * D + c, s0, s1);
    }
    if (threadIdx.x < G) {
      float s = 0.0f, MM = sm_m[threadIdx.x];
#pragma unroll
      for (int w = 0; w < NW; ++w) { s += sm_l[w * 16 + threadIdx.x]; MM = fmaxf(MM, sm_m[w * 16 + threadIdx.x]); }
      st_dev2(pml + threadIdx.x * 2, MM, s);
    }
  }

  // ---- log-sum-exp merge of this head's splits, by the block that finishes last ----
  if (split == 0) FKV_ASTAMP(18);
  if (!last_block_done(a.counters + head, a.n_splits)) return;
  FKV_ASTAMP(19);
  // Every thread owns two output channels of one head and folds that head's splits with an
  // online log-sum-exp.  The (m, l) pairs and the partial outputs of up to CH splits are all
  // requested before the first one is used: one memory round trip per CH splits, no LDS.  CH is
  // matched to the number of splits: a trip issues 2 x CH device-scope loads per thread whether
  // the splits exist or not.
  const size_t pbase = (size_t)head * a.max_splits;
  const int nt = NW * 64, items = G * D / 2;
  auto merge = [&](auto chc) {
  constexpr int CH = decltype(chc)::value;
  for (int it = threadIdx.x; it < items; it += nt) {
    const int gg = it / (D / 2), c2 = it % (D / 2);
    const float* src_o = a.part_o + (pbase * G + gg) * D + c2 * 2;
    const float* src_ml = a.part_ml + (pbase * G + gg) * 2;
    float M = -__builtin_inff(), den = 0.0f, o0 = 0.0f, o1 = 0.0f;
    for (int s0 = 0; s0 < a.n_splits; s0 += CH) {
      float2 ml[CH], v[CH];
#pragma unroll
      for (int u = 0; u < CH; ++u) {
        const int sp = min(s0 + u, a.n_splits - 1);
        ml[u] = ld_dev2(src_ml + (size_t)sp * G * 2);
        v[u] = ld_dev2(src_o + (size_t)sp * G * D);
      }
      float Mc = M;
#pragma unroll
      for (int u = 0; u < CH; ++u)
        if (s0 + u < a.n_splits) Mc = fmaxf(Mc, ml[u].x);
      const float resc = (M == -__builtin_inff()) ? 0.0f : fast_exp2(M - Mc);
      den *= resc; o0 *= resc; o1 *= resc;
      M = Mc;
#pragma unroll
      for (int u = 0; u < CH; ++u) {
        const float w = (s0 + u < a.n_splits && ml[u].x != -__builtin_inff()) ? fast_exp2(ml[u].x - M) : 0.0f;
        den += w * ml[u].y;
        o0 += w * v[u].x;
        o1 += w * v[u].y;
      }
    }
    const float inv = 1.0f / den;
    *reinterpret_cast<float2*>(a.out + (size_t)(b * n_q + m * G + gg) * D + c2 * 2) = make_float2(o0 * inv, o1 * inv);
  }
  };
  if (a.n_splits <= 4) merge(MergeChunk<4>{});
  else if (a.n_splits <= 8) merge(MergeChunk<8>{});
  else if (a.n_splits <= 12) merge(MergeChunk<12>{});
  else if (a.n_splits <= 16) merge(MergeChunk<16>{});
  else if (a.n_splits <= 24) merge(MergeChunk<24>{});
  else merge(MergeChunk<32>{});
  FKV_ASTAMP(21);
#ifdef FKV_SEL_STAMPS
  if (a.tstamp && threadIdx.x == 0) a.tstamp[32 + (head & 7)] = wall_clock64();
#endif
#undef FKV_ASTAMP
}

}  // namespace fkv
