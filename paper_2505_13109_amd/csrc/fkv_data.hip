// Data-plane kernels: bulk context load, summary recompute, page offload to / recall from the host pool.
#include "fkv_device.h"

namespace fkv {

// ---- bulk load: grid (n_pages, n_kv, batch), 256 threads ------------------------
template <int DT>
__global__ __launch_bounds__(256) void load_prefix_kernel(PoolDesc pd, uint16_t* __restrict__ summ,
                                                          uint16_t* __restrict__ host_pool,
                                                          const uint16_t* __restrict__ K,
                                                          const uint16_t* __restrict__ V, int n_tokens,
                                                          int n_kv, int max_pages) {
  __shared__ __attribute__((aligned(16))) uint16_t sk[PG * D];
  __shared__ __attribute__((aligned(16))) uint16_t sv[PG * D];
  const int page = blockIdx.x, m = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
  const int n_pages = (n_tokens + PG - 1) / PG;
  const int nv = min(PG, n_tokens - page * PG);
  for (int i = tid; i < PG * D / 8; i += 256) {
    const int t = i >> 4, c8 = i & 15;
    uint4 kv4 = make_uint4(0, 0, 0, 0), vv4 = make_uint4(0, 0, 0, 0);
    if (t < nv) {
      const size_t src = ((size_t)(b * (size_t)n_tokens + page * PG + t) * n_kv + m) * D + c8 * 8;
      kv4 = *reinterpret_cast<const uint4*>(K + src);
      vv4 = *reinterpret_cast<const uint4*>(V + src);
    }
    *reinterpret_cast<uint4*>(sk + t * D + c8 * 8) = kv4;
    *reinterpret_cast<uint4*>(sv + t * D + c8 * 8) = vv4;
  }
  __syncthreads();
  // destinations: the HBM unit (if this page is resident there) and the host pool unit
  uint16_t* dst_gpu = nullptr;
  uint16_t* dst_host = nullptr;
  if (pd.placement == 0) {
    dst_gpu = pd.pool + (head_base(pd, b, m, n_kv) + page) * UNIT_ELEMS;
  } else {
    if (page < pd.ring_base || page >= n_pages - pd.n_ring)
      dst_gpu = pd.pool + (head_base(pd, b, m, n_kv) + resident_unit(pd, page)) * UNIT_ELEMS;
    dst_host = host_pool + ((size_t)(b * n_kv + m) * max_pages + page) * UNIT_ELEMS;
  }
  for (int i = tid; i < UNIT_ELEMS / 8; i += 256) {
    __attribute__((aligned(16))) uint16_t o[8];
    if (i < PG * D / 8) {   // K page: 8 consecutive channels of one token
      const int mm = i & 15, kb = (i >> 4) & 3, j8 = i >> 6;
      const int t = (j8 & 1) * 16 + mm, ch0 = ((j8 >> 1) * 4 + kb) * 8;
      *reinterpret_cast<uint4*>(o) = *reinterpret_cast<const uint4*>(sk + t * D + ch0);
    } else {                // V page: one channel of 8 tokens
      const int iv = i - PG * D / 8;
      const int mm = iv & 15, kb = (iv >> 4) & 3, cb = iv >> 6;
      const int ch = cb * 16 + mm;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int t = (e < 4) ? kb * 4 + e : 16 + kb * 4 + (e - 4);
        o[e] = sv[t * D + ch];
      }
    }
    const uint4 w = *reinterpret_cast<const uint4*>(o);
    if (dst_gpu) *reinterpret_cast<uint4*>(dst_gpu + i * 8) = w;
    if (dst_host) *reinterpret_cast<uint4*>(dst_host + i * 8) = w;
  }
  if (tid < D) {
    uint16_t bmax = sk[tid], bmin = sk[tid];
    float fmax_ = Unpack<DT>::one(bmax), fmin_ = fmax_;
    for (int t = 1; t < nv; ++t) {
      const uint16_t kb = sk[t * D + tid];
      const float kf = Unpack<DT>::one(kb);
      if (kf > fmax_) { fmax_ = kf; bmax = kb; }
      if (kf < fmin_) { fmin_ = kf; bmin = kb; }
    }
    summ[summ_idx(b, m, n_kv, 0, max_pages, page) + tid] = bmax;
    summ[summ_idx(b, m, n_kv, 1, max_pages, page) + tid] = bmin;
  }
}

// ---- recompute summaries from stored keys (placement HBM): grid (n_pages, n_kv, batch), 128 threads
template <int DT>
__global__ __launch_bounds__(128) void summary_recompute_kernel(PoolDesc pd, uint16_t* __restrict__ summ,
                                                                int first_page, Geom g, int n_kv,
                                                                int max_pages) {
  const int page = first_page + blockIdx.x, m = blockIdx.y, b = blockIdx.z, c = threadIdx.x;
  const int nv = page < g.n_full ? PG : (page == g.n_full ? g.r : 0);
  if (nv == 0) return;
  const uint16_t* unit = pd.pool + (head_base(pd, b, m, n_kv) + page) * UNIT_ELEMS;
  uint16_t bmax = unit[k_elem_off(0, c)], bmin = bmax;
  float fmax_ = Unpack<DT>::one(bmax), fmin_ = fmax_;
  for (int t = 1; t < nv; ++t) {
    const uint16_t kb = unit[k_elem_off(t, c)];
    const float kf = Unpack<DT>::one(kb);
    if (kf > fmax_) { fmax_ = kf; bmax = kb; }
    if (kf < fmin_) { fmin_ = kf; bmin = kb; }
  }
  summ[summ_idx(b, m, n_kv, 0, max_pages, page) + c] = bmax;
  summ[summ_idx(b, m, n_kv, 1, max_pages, page) + c] = bmin;
}

// ---- offload a filled page to the host pool: grid (n_kv, batch), 256 threads ------
__global__ __launch_bounds__(256) void offload_kernel(PoolDesc pd, uint16_t* __restrict__ host_pool,
                                                      int page, int n_kv, int max_pages) {
  const int m = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const uint4* src = reinterpret_cast<const uint4*>(
      pd.pool + (head_base(pd, b, m, n_kv) + resident_unit(pd, page)) * UNIT_ELEMS);
  uint4* dst = reinterpret_cast<uint4*>(host_pool + ((size_t)(b * n_kv + m) * max_pages + page) * UNIT_ELEMS);
  uint4 w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = src[tid + i * 256];
#pragma unroll
  for (int i = 0; i < 4; ++i) dst[tid + i * 256] = w[i];
}

// ---- recall: copy missing pages host pool -> free page-cache slots ---------------
// miss: [heads][1 + 2k] = count, then k page ids, then k slots.
// A few 1024-thread blocks share the miss lists, four 16 KiB units in flight per block.  Loads
// from host memory take microseconds to return and hold up the memory pipeline of the compute
// unit they are issued from, so the blocks are kept few and each one claims a whole compute
// unit's LDS: no block of a kernel that uses LDS (attention, scoring) can share that unit.
constexpr int GATHER_THREADS = 1024;
constexpr int GATHER_BLOCKS = 16;            // measured: 8 and 16 blocks move 52-53 GB/s, 24 blocks 50, 32 blocks 47
constexpr int GATHER_UNITS = 4;              // units in flight per block (8 is no faster)
__global__ __launch_bounds__(GATHER_THREADS) void gather_kernel(PoolDesc pd, const uint16_t* __restrict__ host_pool,
                                                                const int32_t* __restrict__ miss,
                                                                const uint8_t* __restrict__ flags, int heads_mode,
                                                                int k, int n_kv, int n_heads, int max_pages) {
  extern __shared__ int32_t chunks_of[];     // [n_heads]: 4-unit chunks this launch moves for each head
  const int tid = threadIdx.x;
  // The chunks (GATHER_UNITS units each) of all chosen heads, numbered through, are dealt to the blocks in turn, so that every
  // block moves the same amount whatever the heads' miss counts are (a corrected-heads launch
  // serves about every other head, with anything from 0 to k misses).
  for (int head = tid; head < n_heads; head += GATHER_THREADS) {
    const bool chosen = heads_mode == 0 || ((heads_mode == 1) == (flags[head] != 0));
    chunks_of[head] = chosen ? (miss[(size_t)head * (1 + 2 * k)] + GATHER_UNITS - 1) / GATHER_UNITS : 0;
  }
  __syncthreads();
  int first = 0;                                // number of the head's first chunk
  for (int head = 0; head < n_heads; ++head) {
    const int n_chunks = chunks_of[head];
    const int c_begin = first;
    first += n_chunks;
    // chunks of this head that are this block's: c_begin + j with (c_begin + j) % gridDim.x == blockIdx.x
    int j = ((int)blockIdx.x - c_begin % (int)gridDim.x + (int)gridDim.x) % (int)gridDim.x;
    if (j >= n_chunks) continue;
    const int32_t* mh = miss + (size_t)head * (1 + 2 * k);
    const int n = mh[0];
    const uint16_t* src_head = host_pool + (size_t)head * max_pages * UNIT_ELEMS;
    uint16_t* dst_head = pd.pool + ((size_t)head * pd.units_per_head + pd.sel_base) * UNIT_ELEMS;
    for (; j < n_chunks; j += gridDim.x) {
      const int i0 = j * GATHER_UNITS;
      uint4 w[GATHER_UNITS];
#pragma unroll
      for (int u = 0; u < GATHER_UNITS; ++u) {
        const int i = min(i0 + u, n - 1);
        w[u] = reinterpret_cast<const uint4*>(src_head + (size_t)mh[1 + i] * UNIT_ELEMS)[tid];
      }
#pragma unroll
      for (int u = 0; u < GATHER_UNITS; ++u) {
        if (i0 + u < n) reinterpret_cast<uint4*>(dst_head + (size_t)mh[1 + k + i0 + u] * UNIT_ELEMS)[tid] = w[u];
      }
    }
  }
}

// ---- recall plan: which picked pages are already cached, where the others go ------
// A page hits iff it is in the ACTIVE selection (it keeps that slot).  Misses go, in
// ascending page order, to the lowest-numbered slots the ACTIVE selection does not use.
// grid (n_kv, batch), 64 threads (one wave); pool of 2k slots per head; k <= 1024.
// An id that is not a full page of the context (a caller's list may hold anything) is dropped:
// rewritten to -1 in new_ids, so that neither the gather nor attention ever forms its address.
__global__ __launch_bounds__(64) void plan_kernel(int32_t* __restrict__ new_ids,
                                                  const int32_t* __restrict__ act_ids,
                                                  const int32_t* __restrict__ act_slots,
                                                  int32_t* __restrict__ new_slots,
                                                  int32_t* __restrict__ miss, int k, int n_kv, int n_full) {
  extern __shared__ int32_t sm[];          // used[2k], aid[k], aslot[k], nid[k], nslot[k], freelist[2k]
  int32_t* used = sm;
  int32_t* aid = sm + 2 * k;
  int32_t* aslot = aid + k;
  int32_t* nid = aslot + k;
  int32_t* nslot = nid + k;
  int32_t* freelist = nslot + k;
  const int m = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
  const size_t hb = (size_t)(b * n_kv + m) * k;
  int32_t* mh = miss + (size_t)(b * n_kv + m) * (1 + 2 * k);
  for (int s = lane; s < 2 * k; s += 64) used[s] = 0;
  int n_act = 0;
  for (int i = lane; i < k; i += 64) {     // all lists in one round trip
    aid[i] = act_ids[hb + i];
    aslot[i] = act_slots[hb + i];
    const int32_t id = new_ids[hb + i];
    nid[i] = id < n_full ? id : -1;
    if (id >= n_full) new_ids[hb + i] = -1;
  }
  __syncthreads();
  for (int i = lane; i < k; i += 64) {
    if (aid[i] >= 0) { used[aslot[i]] = 1; ++n_act; }
  }
  n_act = (int)wave_sum_u32((uint32_t)n_act);   // ids are ascending, -1 padded at the end
  __syncthreads();
  // hit or miss per picked page (binary search in the ACTIVE ids)
  for (int i = lane; i < k; i += 64) {
    const int id = nid[i];
    int slot = -1;
    if (id >= 0) {
      int lo = 0, hi = n_act;
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (aid[mid] < id) lo = mid + 1; else hi = mid;
      }
      slot = (lo < n_act && aid[lo] == id) ? aslot[lo] : -2;   // -2: miss
    }
    nslot[i] = slot;
  }
  // ordered list of free slots
  int base = 0;
  for (int s0 = 0; s0 < 2 * k; s0 += 64) {
    const int s = s0 + lane;
    const uint32_t f = (s < 2 * k && !used[s]) ? 1u : 0u;
    const uint32_t incl = wave_scan_u32(f);
    if (f) freelist[base + (int)incl - 1] = s;
    base += (int)__builtin_amdgcn_readlane((int)incl, 63);
  }
  __syncthreads();
  // the r-th miss (ascending page id) takes the r-th free slot
  int n_miss = 0;
  for (int i0 = 0; i0 < k; i0 += 64) {
    const int i = i0 + lane;
    const uint32_t f = (i < k && nslot[i] == -2) ? 1u : 0u;
    const uint32_t incl = wave_scan_u32(f);
    if (f) {
      const int r = n_miss + (int)incl - 1;
      const int s = freelist[r];
      nslot[i] = s;
      mh[1 + r] = nid[i];
      mh[1 + k + r] = s;
    }
    n_miss += (int)__builtin_amdgcn_readlane((int)incl, 63);
  }
  if (lane == 0) mh[0] = n_miss;
  __syncthreads();
  for (int i = lane; i < k; i += 64) new_slots[hb + i] = nslot[i];
}

// ---- debug: one unit -> token-major K [p, d], V [p, d] ---------------------------
__global__ __launch_bounds__(256) void read_page_kernel(const uint16_t* __restrict__ unit,
                                                        uint16_t* __restrict__ out) {
  for (int i = threadIdx.x; i < PG * D; i += 256) {
    const int t = i / D, c = i % D;
    out[i] = unit[k_elem_off(t, c)];
    out[PG * D + i] = unit[v_elem_off(t, c)];
  }
}

// ---- launch wrappers ----------------------------------------------------------------
void launch_load_prefix(const Dims& d, const PoolDesc& pd, uint16_t* summ, uint16_t* host_pool,
                        const uint16_t* K, const uint16_t* V, int n_tokens, Geom g, hipStream_t st) {
  (void)g;
  const int n_pages = (n_tokens + PG - 1) / PG;
  if (n_pages == 0) return;
  dim3 grid(n_pages, d.n_kv, d.batch);
  if (d.dtype == 0) load_prefix_kernel<0><<<grid, 256, 0, st>>>(pd, summ, host_pool, K, V, n_tokens, d.n_kv, d.max_pages);
  else              load_prefix_kernel<1><<<grid, 256, 0, st>>>(pd, summ, host_pool, K, V, n_tokens, d.n_kv, d.max_pages);
}

void launch_summary_recompute(const Dims& d, const PoolDesc& pd, uint16_t* summ, int first_page,
                              int n_pages, Geom g, hipStream_t st) {
  if (n_pages <= 0) return;
  dim3 grid(n_pages, d.n_kv, d.batch);
  if (d.dtype == 0) summary_recompute_kernel<0><<<grid, 128, 0, st>>>(pd, summ, first_page, g, d.n_kv, d.max_pages);
  else              summary_recompute_kernel<1><<<grid, 128, 0, st>>>(pd, summ, first_page, g, d.n_kv, d.max_pages);
}

void launch_offload(const Dims& d, const PoolDesc& pd, uint16_t* host_pool, int page, hipStream_t st) {
  dim3 grid(d.n_kv, d.batch);
  offload_kernel<<<grid, 256, 0, st>>>(pd, host_pool, page, d.n_kv, d.max_pages);
}

void launch_plan(const Dims& d, int32_t* new_ids, const int32_t* act_ids, const int32_t* act_slots,
                 int32_t* new_slots, int32_t* miss, int n_full, hipStream_t st) {
  if (d.k == 0) return;
  dim3 grid(d.n_kv, d.batch);
  plan_kernel<<<grid, 64, 8 * d.k * sizeof(int32_t), st>>>(new_ids, act_ids, act_slots, new_slots, miss, d.k, d.n_kv, n_full);
}

void launch_gather(const Dims& d, const PoolDesc& pd, const uint16_t* host_pool, const int32_t* miss,
                   const int32_t*, const uint8_t* flags, int heads, hipStream_t st) {
  if (d.k == 0) return;
  static bool raised = false;
  const int hog = d.max_lds > 64 * 1024 ? d.max_lds - 1024 : 64 * 1024 - 1024;   // (nearly) all of a unit's LDS
  if (!raised) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gather_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, hog);
    (void)hipGetLastError();
    raised = true;
  }
  const int n_heads = d.batch * d.n_kv;
  const int blocks = n_heads < GATHER_BLOCKS ? n_heads : GATHER_BLOCKS;
  gather_kernel<<<blocks, GATHER_THREADS, hog, st>>>(pd, host_pool, miss, flags, heads, d.k, d.n_kv, n_heads, d.max_pages);
}

void launch_read_page(const uint16_t* unit, uint16_t* out_token_major, hipStream_t st) {
  read_page_kernel<<<1, 256, 0, st>>>(unit, out_token_major);
}

}  // namespace fkv
