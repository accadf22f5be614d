// Stand-alone launch of sparse decode attention (device code in fkv_attn_dev.h).
#include "fkv_attn_dev.h"

namespace fkv {

// grid (n_splits, n_kv, batch); NW wavefronts per block
template <int DT, int NW>
__global__ __launch_bounds__(NW * 64) void attn_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) float lds[NW > 1 ? NW * (32 + MAX_G * D) : 1];
  attn_block<DT, NW>(a, blockIdx.x, blockIdx.y, blockIdx.z, lds);
}

// experiment builds only (see knob()): pages per block (0 = choose from the shape)
static const int g_pps_override = knob("FKV_ATTN_PPS", 0);

// pages per block of NW waves for a head with n_att attended pages
int attn_pages_per_block(int n_att, int heads, int max_splits, int nw) {
  // a page per wave and pass; more pages per block (the page loop is pipelined, the merge gets
  // cheaper) as long as the launch keeps at least ~128 blocks, and never more than 32 splits
  // per KV head beyond that, so that the merge needs one round trip
  int pps = nw;
  while (pps < 16 && (long)heads * ((n_att + pps * 2 - 1) / (pps * 2)) >= 128) pps *= 2;
  while ((n_att + pps - 1) / pps > 32 && (long)heads * ((n_att + pps * 2 - 1) / (pps * 2)) >= 128) pps *= 2;
  // With many heads the launch is bandwidth-bound and what counts is the fixed cost of a block
  // (its partial, the counter, the merge): measured best at about one block per compute unit,
  // down to one block per head.
  while (pps < n_att && (long)heads * ((n_att + pps * 2 - 1) / (pps * 2)) >= 256) pps *= 2;
  while ((n_att + pps - 1) / pps > (max_splits < MAX_MERGE_SPLITS ? max_splits : MAX_MERGE_SPLITS)) pps *= 2;
  if (pps > 16) {                                   // long blocks: split the head evenly
    const int n_splits = (n_att + pps - 1) / pps;
    pps = (n_att + n_splits - 1) / n_splits;
  }
  if (g_pps_override > 0) pps = g_pps_override;
  return pps;
}

int launch_attn(const Dims& d, const PoolDesc& pd, const uint16_t* q, const int32_t* act_ids,
                const int32_t* new_ids, const int32_t* act_slots, const int32_t* new_slots,
                const uint8_t* flags, int use, float* part_o, float* part_ml, int max_splits,
                int* counters, float* out, Geom g, hipStream_t st, hipEvent_t ev_begin, hipEvent_t ev_end,
                long long* tstamp) {
  const int n_att = g.n_sink + d.k + g.n_win + (g.r > 0 ? 1 : 0);
  AttnArgs a{};
  a.pd = pd; a.q = q; a.act_ids = act_ids; a.new_ids = new_ids; a.act_slots = act_slots; a.new_slots = new_slots;
  a.flags = flags; a.use = use; a.part_o = part_o; a.part_ml = part_ml; a.max_splits = max_splits;
  a.pps = attn_pages_per_block(n_att, d.n_kv * d.batch, max_splits, 4);
  a.n_splits = (n_att + a.pps - 1) / a.pps;
  a.counters = counters; a.out = out; a.g = g; a.n_q = d.n_q; a.n_kv = d.n_kv; a.G = d.G; a.k = d.k;
  a.tstamp = tstamp; a.fused = 0;
  const int nw = a.pps >= 4 ? 4 : a.pps;
  dim3 grid(a.n_splits, d.n_kv, d.batch);
  if (ev_begin) (void)hipEventRecord(ev_begin, st);
  if (d.dtype == 0) {
    if (nw == 1)      attn_kernel<0, 1><<<grid, 64, 0, st>>>(a);
    else if (nw == 2) attn_kernel<0, 2><<<grid, 128, 0, st>>>(a);
    else              attn_kernel<0, 4><<<grid, 256, 0, st>>>(a);
  } else {
    if (nw == 1)      attn_kernel<1, 1><<<grid, 64, 0, st>>>(a);
    else if (nw == 2) attn_kernel<1, 2><<<grid, 128, 0, st>>>(a);
    else              attn_kernel<1, 4><<<grid, 256, 0, st>>>(a);
  }
  if (ev_end) (void)hipEventRecord(ev_end, st);
  return a.n_splits;
}

__global__ __launch_bounds__(256) void fill_zero_kernel(int* __restrict__ p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}
void launch_fill_zero(int* p, int n, hipStream_t st) {
  if (n > 0) fill_zero_kernel<<<(n + 255) / 256, 256, 0, st>>>(p, n);
}

// ---------------------------------------------------------------------------------
// The pages a head attends, converted to the NHD layout of the paper's hybrid layouts
// (Sec. 4.2): out [batch][n_slots][2 (K, V)][page][n_kv][d], slot s of head m = position s of
// m's attend list; slot_pages [batch][n_kv][n_slots].  One block per (slot, head): the 16 KiB
// unit comes in with linear 16-byte loads, is turned in LDS, and goes out as 256-byte token rows.
// ---------------------------------------------------------------------------------
// `miss` (may be null): the recall plan's miss lists [heads][1 + 3k].  With it, a picked page that the
// plan marked missing is left alone -- its rows arrive through the streamed recall -- and only its
// page id is recorded.
__global__ __launch_bounds__(256) void export_nhd_kernel(AttnArgs a, uint16_t* __restrict__ out,
                                                         int32_t* __restrict__ slot_pages, int n_slots,
                                                         const int32_t* __restrict__ miss) {
  __shared__ __attribute__((aligned(16))) uint16_t unit_lds[UNIT_ELEMS];
  __shared__ int s_missing;
  const int slot = blockIdx.x, m = blockIdx.y, b = blockIdx.z;
  const int head = b * a.n_kv + m, k = a.k;
  const Geom& g = a.g;
  const bool pending = a.use == 1 || (a.use == 2 && a.flags[head] != 0);
  AttendList al;
  al.ids = (pending ? a.new_ids : a.act_ids) + (size_t)head * k;
  al.slots = a.pd.placement == 0 ? nullptr : (pending ? a.new_slots : a.act_slots) + (size_t)head * k;
  al.n_sink = g.n_sink; al.k = k; al.n_win = g.n_win; al.n_full = g.n_full; al.r = g.r;
  al.coherent_ids = false;
  const int n_att = g.n_sink + k + g.n_win + (g.r > 0 ? 1 : 0);
  int n_valid = 0, page = -1, unit = -1;
  if (slot < n_att) unit = attend_unit(al, a.pd, slot, n_valid, page);
  if (unit < 0) { page = -1; n_valid = 0; }
  if (threadIdx.x == 0) slot_pages[(size_t)head * n_slots + slot] = page;
  if (miss && unit >= 0 && slot >= g.n_sink && slot < g.n_sink + k) {
    if (threadIdx.x == 0) s_missing = 0;
    __syncthreads();
    const int32_t* mh = miss + (size_t)head * (1 + 3 * k);
    for (int r = threadIdx.x; r < mh[0]; r += 256)
      if (mh[1 + 2 * k + r] == slot - g.n_sink) s_missing = 1;
    __syncthreads();
    if (s_missing) return;
  }
  if (unit >= 0) {
    const uint4* src = reinterpret_cast<const uint4*>(a.pd.pool + ((size_t)head * a.pd.units_per_head + unit) * UNIT_ELEMS);
    uint4* dst = reinterpret_cast<uint4*>(unit_lds);
#pragma unroll
    for (int i = 0; i < UNIT_ELEMS / 8 / 256; ++i) dst[threadIdx.x + i * 256] = src[threadIdx.x + i * 256];
  }
  __syncthreads();
  // 2 x 32 token rows of 16 chunks of 8 channels
  for (int i = threadIdx.x; i < 2 * PG * (D / 8); i += 256) {
    const int c8 = i % (D / 8), t = (i / (D / 8)) % PG, kv = i / (D / 8) / PG;
    uint4 w = make_uint4(0, 0, 0, 0);
    if (t < n_valid) {
      if (kv == 0) {
        w = *reinterpret_cast<const uint4*>(unit_lds + k_elem_off(t, c8 * 8));    // 8 channels lie together
      } else {
        uint16_t e[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) e[c] = unit_lds[v_elem_off(t, c8 * 8 + c)];
        w.x = e[0] | ((uint32_t)e[1] << 16); w.y = e[2] | ((uint32_t)e[3] << 16);
        w.z = e[4] | ((uint32_t)e[5] << 16); w.w = e[6] | ((uint32_t)e[7] << 16);
      }
    }
    uint16_t* row = out + ((((size_t)(b * n_slots + slot) * 2 + kv) * PG + t) * a.n_kv + m) * D;
    *reinterpret_cast<uint4*>(row + c8 * 8) = w;
  }
}

void launch_export_nhd(const Dims& d, const PoolDesc& pd, const int32_t* act_ids, const int32_t* new_ids,
                       const int32_t* act_slots, const int32_t* new_slots, const uint8_t* flags, int use,
                       uint16_t* out, int32_t* slot_pages, int n_slots, Geom g, hipStream_t st, const int32_t* skip_missing) {
  AttnArgs a{};
  a.pd = pd; a.act_ids = act_ids; a.new_ids = new_ids; a.act_slots = act_slots; a.new_slots = new_slots;
  a.flags = flags; a.use = use; a.g = g; a.n_q = d.n_q; a.n_kv = d.n_kv; a.G = d.G; a.k = d.k;
  dim3 grid(n_slots, d.n_kv, d.batch);
  export_nhd_kernel<<<grid, 256, 0, st>>>(a, out, slot_pages, n_slots, skip_missing);
}

}  // namespace fkv
