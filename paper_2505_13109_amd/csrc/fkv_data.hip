// Data-plane kernels: bulk context load, summary recompute, page offload to / recall from the host pool.
#include "fkv_device.h"
#include "fkv_plan_dev.h"

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
// miss: [heads][1 + 3k] = count, then k page ids, k slots, k positions in the picked list.
// A few 1024-thread blocks share the miss lists, four 16 KiB units in flight per block.  Loads
// from host memory take microseconds to return and hold up the memory pipeline of the compute
// unit they are issued from, so the blocks are kept few and each one claims a whole compute
// unit's LDS: no block of a kernel that uses LDS (attention, scoring) can share that unit.
constexpr int GATHER_THREADS = 1024;
constexpr int GATHER_BLOCKS = 16;            // measured: 8 and 16 blocks move 52-53 GB/s, 24 blocks 50, 32 blocks 47
constexpr int GATHER_UNITS = 4;              // units in flight per block (8 is no faster)
// One launch serves the miss lists of up to GATHER_MAX_LAYERS layers (the deferred recall of several layers is
// submitted together); a "head" below is a (layer, KV head) pair, numbered layer-major.
__global__ __launch_bounds__(GATHER_THREADS) void gather_kernel(GatherLayers gl, int heads_mode,
                                                                int k, int n_kv, int n_heads, int max_pages) {
  extern __shared__ int32_t chunks_of[];     // [n_layers * n_heads]: 4-unit chunks this launch moves for each head
  const int tid = threadIdx.x;
  const int n_all = gl.n * n_heads;
  // The chunks (GATHER_UNITS units each) of all chosen heads, numbered through, are dealt to the blocks in turn, so that every
  // block moves the same amount whatever the heads' miss counts are (a corrected-heads launch
  // serves about every other head, with anything from 0 to k misses).
  for (int h = tid; h < n_all; h += GATHER_THREADS) {
    const int li = h / n_heads, head = h % n_heads;
    const bool chosen = heads_mode == 0 || ((heads_mode == 1) == (gl.flags[li][head] != 0));
    chunks_of[h] = chosen ? (gl.miss[li][(size_t)head * (1 + 3 * k)] + GATHER_UNITS - 1) / GATHER_UNITS : 0;
  }
  __syncthreads();
  int first = 0;                                // number of the head's first chunk
  for (int h = 0; h < n_all; ++h) {
    const int n_chunks = chunks_of[h];
    const int c_begin = first;
    first += n_chunks;
    // chunks of this head that are this block's: c_begin + j with (c_begin + j) % gridDim.x == blockIdx.x
    int j = ((int)blockIdx.x - c_begin % (int)gridDim.x + (int)gridDim.x) % (int)gridDim.x;
    if (j >= n_chunks) continue;
    const int li = h / n_heads, head = h % n_heads;
    const PoolDesc& pd = gl.pd[li];
    const int32_t* mh = gl.miss[li] + (size_t)head * (1 + 3 * k);
    const int n = mh[0];
    const uint16_t* src_head = gl.host_pool[li] + (size_t)head * max_pages * UNIT_ELEMS;
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

// ---- streamed recall into an NHD pool (Sec. 4.2 "Hybrid layouts", "Streamed recall") -------------
// The paper keeps the GPU pool in NHD (tokens with all KV heads side by side) and the host pool in
// per-(page, head) units; a recalled unit is turned into NHD on its way in, through two staging
// buffers, so that the transfer of one unit overlaps the conversion of the previous one.  Here the
// staging buffers are two LDS buffers of GATHER_UNITS units per block: while the block turns the
// units of buffer A into 256-byte token rows of the pool, the loads of its next units from the
// pinned host pool are already in flight, and land in buffer B.  The unit also goes, unconverted,
// to its page-cache slot (what this library's own attention reads, and what makes the page a hit
// at the next step).  nhd: [batch][n_slots][2 (K, V)][PG][n_kv][D]; a miss at position i of its
// head's picked list goes to pool slot n_sink + i.
__global__ __launch_bounds__(GATHER_THREADS) void gather_nhd_kernel(PoolDesc pd, const uint16_t* __restrict__ host_pool,
                                                                    const int32_t* __restrict__ miss,
                                                                    const uint8_t* __restrict__ flags, int heads_mode,
                                                                    int k, int n_kv, int n_heads, int max_pages,
                                                                    uint16_t* __restrict__ nhd, int n_slots, int n_sink) {
  extern __shared__ __attribute__((aligned(16))) unsigned char gsm[];
  uint16_t* stage = reinterpret_cast<uint16_t*>(gsm);                                   // [2][GATHER_UNITS][UNIT_ELEMS]
  int32_t* chunks_of = reinterpret_cast<int32_t*>(gsm + 2 * GATHER_UNITS * UNIT_BYTES);   // [n_heads]
  const int tid = threadIdx.x;
  for (int head = tid; head < n_heads; head += GATHER_THREADS) {
    const bool chosen = heads_mode == 0 || ((heads_mode == 1) == (flags[head] != 0));
    chunks_of[head] = chosen ? (miss[(size_t)head * (1 + 3 * k)] + GATHER_UNITS - 1) / GATHER_UNITS : 0;
  }
  __syncthreads();
  // this block's chunks, in order: chunk c of the launch-wide numbering is ours iff c % gridDim.x == blockIdx.x
  struct Cursor { int head, first, j; };          // head, number of its first chunk, chunk within the head
  auto advance = [&](Cursor& c) -> bool {         // to this block's next chunk; false when there is none
    for (;;) {
      if (c.head >= n_heads) return false;
      const int n_chunks = chunks_of[c.head];
      if (c.j < 0) c.j = ((int)blockIdx.x - c.first % (int)gridDim.x + (int)gridDim.x) % (int)gridDim.x;
      else c.j += gridDim.x;
      if (c.j < n_chunks) return true;
      c.first += n_chunks;
      c.head += 1;
      c.j = -1;
    }
  };
  auto load = [&](const Cursor& c, uint4* w) {
    const int32_t* mh = miss + (size_t)c.head * (1 + 3 * k);
    const int n = mh[0];
    const uint16_t* src_head = host_pool + (size_t)c.head * max_pages * UNIT_ELEMS;
#pragma unroll
    for (int u = 0; u < GATHER_UNITS; ++u) {
      const int i = min(c.j * GATHER_UNITS + u, n - 1);
      w[u] = reinterpret_cast<const uint4*>(src_head + (size_t)mh[1 + i] * UNIT_ELEMS)[tid];
    }
  };
  Cursor cur{0, 0, -1};
  bool have = advance(cur);
  uint4 w[GATHER_UNITS];
  if (have) load(cur, w);
  int buf = 0;
  while (have) {
    const int32_t* mh = miss + (size_t)cur.head * (1 + 3 * k);
    const int n = mh[0], i0 = cur.j * GATHER_UNITS;
    uint16_t* dst_head = pd.pool + ((size_t)cur.head * pd.units_per_head + pd.sel_base) * UNIT_ELEMS;
    uint16_t* st_buf = stage + (size_t)buf * GATHER_UNITS * UNIT_ELEMS;
#pragma unroll
    for (int u = 0; u < GATHER_UNITS; ++u) {
      if (i0 + u < n) {
        reinterpret_cast<uint4*>(dst_head + (size_t)mh[1 + k + i0 + u] * UNIT_ELEMS)[tid] = w[u];    // page-cache slot
        reinterpret_cast<uint4*>(st_buf + (size_t)u * UNIT_ELEMS)[tid] = w[u];                         // staging buffer
      }
    }
    // the next chunk's transfer starts now and runs during the conversion below
    const Cursor done = cur;
    have = advance(cur);
    if (have) load(cur, w);
    __syncthreads();
    // conversion: unit u of the staging buffer -> 2 x PG token rows of 16 chunks of 8 channels
    const int b = done.head / n_kv, m = done.head % n_kv;
#pragma unroll
    for (int u = 0; u < GATHER_UNITS; ++u) {
      if (i0 + u >= n) break;
      const int slot = n_sink + mh[1 + 2 * k + i0 + u];
      const uint16_t* unit = st_buf + (size_t)u * UNIT_ELEMS;
      for (int i = tid; i < 2 * PG * (D / 8); i += GATHER_THREADS) {
        const int c8 = i % (D / 8), t = (i / (D / 8)) % PG, kv = i / (D / 8) / PG;
        uint4 o;
        if (kv == 0) {
          o = *reinterpret_cast<const uint4*>(unit + k_elem_off(t, c8 * 8));        // 8 channels lie together
        } else {
          uint16_t e[8];
#pragma unroll
          for (int c = 0; c < 8; ++c) e[c] = unit[v_elem_off(t, c8 * 8 + c)];
          o.x = e[0] | ((uint32_t)e[1] << 16); o.y = e[2] | ((uint32_t)e[3] << 16);
          o.z = e[4] | ((uint32_t)e[5] << 16); o.w = e[6] | ((uint32_t)e[7] << 16);
        }
        uint16_t* row = nhd + ((((size_t)(b * n_slots + slot) * 2 + kv) * PG + t) * n_kv + m) * D;
        *reinterpret_cast<uint4*>(row + c8 * 8) = o;
      }
    }
    buf ^= 1;      // the buffer just converted is written again two chunks on, behind the next barrier
  }
}

// ---- recall plan (fkv_plan_dev.h) as a launch of its own: grid (n_kv, batch), one wave ------------
__global__ __launch_bounds__(64) void plan_kernel(int32_t* __restrict__ new_ids,
                                                  const int32_t* __restrict__ act_ids,
                                                  const int32_t* __restrict__ act_slots,
                                                  int32_t* __restrict__ new_slots,
                                                  int32_t* __restrict__ miss, int k, int n_kv, int n_full) {
  extern __shared__ int32_t sm[];
  const size_t head = (size_t)blockIdx.y * n_kv + blockIdx.x;
  plan_head<64>(new_ids + head * k, act_ids + head * k, act_slots + head * k, new_slots + head * k,
                miss + head * (1 + 3 * k), k, n_full, sm, false);
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
  plan_kernel<<<grid, 64, plan_lds_ints(d.k) * sizeof(int32_t), st>>>(new_ids, act_ids, act_slots, new_slots, miss, d.k, d.n_kv, n_full);
}

void launch_gather(const Dims& d, const GatherLayers& gl, int heads, hipStream_t st) {
  if (d.k == 0 || gl.n <= 0) return;
  static bool raised = false;
  const int hog = d.max_lds > 64 * 1024 ? d.max_lds - 1024 : 64 * 1024 - 1024;   // (nearly) all of a unit's LDS
  if (!raised) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gather_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, hog);
    (void)hipGetLastError();
    raised = true;
  }
  const int n_heads = d.batch * d.n_kv;
  // the kernel keeps one counter per (layer, head) in LDS: as many layers per launch as fit
  int per_launch = (int)((size_t)hog / sizeof(int32_t) / (size_t)n_heads);
  if (per_launch < 1) per_launch = 1;        // (fkv_create bounds the heads so that one layer always fits)
  for (int l0 = 0; l0 < gl.n; l0 += per_launch) {
    GatherLayers part{};
    part.n = gl.n - l0 < per_launch ? gl.n - l0 : per_launch;
    for (int i = 0; i < part.n; ++i) {
      part.pd[i] = gl.pd[l0 + i]; part.host_pool[i] = gl.host_pool[l0 + i];
      part.miss[i] = gl.miss[l0 + i]; part.flags[i] = gl.flags[l0 + i];
    }
    const int blocks = n_heads * part.n < GATHER_BLOCKS ? n_heads * part.n : GATHER_BLOCKS;
    gather_kernel<<<blocks, GATHER_THREADS, hog, st>>>(part, heads, d.k, d.n_kv, n_heads, d.max_pages);
  }
}

void launch_gather_nhd(const Dims& d, const PoolDesc& pd, const uint16_t* host_pool, const int32_t* miss,
                       const uint8_t* flags, int heads, uint16_t* nhd, int n_slots, int n_sink, hipStream_t st) {
  if (d.k == 0) return;
  static bool raised = false;
  const int n_heads = d.batch * d.n_kv;
  const size_t lds = (size_t)2 * GATHER_UNITS * UNIT_BYTES + (size_t)n_heads * sizeof(int32_t);   // 128 KiB of staging: the unit's LDS is taken anyway
  if (!raised) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gather_nhd_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              d.max_lds > 64 * 1024 ? d.max_lds - 1024 : 64 * 1024 - 1024);
    (void)hipGetLastError();
    raised = true;
  }
  const int blocks = n_heads < GATHER_BLOCKS ? n_heads : GATHER_BLOCKS;
  gather_nhd_kernel<<<blocks, GATHER_THREADS, lds, st>>>(pd, host_pool, miss, flags, heads, d.k, d.n_kv, n_heads, d.max_pages,
                                                          nhd, n_slots, n_sink);
}

void launch_read_page(const uint16_t* unit, uint16_t* out_token_major, hipStream_t st) {
  read_page_kernel<<<1, 256, 0, st>>>(unit, out_token_major);
}

}  // namespace fkv
