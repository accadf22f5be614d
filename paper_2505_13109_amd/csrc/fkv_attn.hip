// Stand-alone launch of sparse decode attention (device code in fkv_attn_dev.h).
#include "fkv_attn_dev.h"
#include <cstdlib>

namespace fkv {

// grid (n_splits, n_kv, batch); NW wavefronts per block
template <int DT, int NW>
__global__ __launch_bounds__(NW * 64) void attn_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) float lds[NW > 1 ? NW * (32 + MAX_G * D) : 1];
  attn_block<DT, NW>(a, blockIdx.x, blockIdx.y, blockIdx.z, lds);
}

// tuning knob for experiments: pages per block (0 = choose from the shape)
static int g_pps_override = [] { const char* e = getenv("FKV_ATTN_PPS"); return e ? atoi(e) : 0; }();

// pages per block of NW waves for a head with n_att attended pages
int attn_pages_per_block(int n_att, int heads, int max_splits, int nw) {
  // a page per wave and pass; more pages per block (the page loop is pipelined, the merge gets
  // cheaper) as long as the launch keeps at least ~128 blocks, and never more than 32 splits
  // per KV head beyond that, so that the merge needs one round trip
  int pps = nw;
  while (pps < 16 && (long)heads * ((n_att + pps * 2 - 1) / (pps * 2)) >= 128) pps *= 2;
  while ((n_att + pps - 1) / pps > 32 && (long)heads * ((n_att + pps * 2 - 1) / (pps * 2)) >= 128) pps *= 2;
  while ((n_att + pps - 1) / pps > (max_splits < MAX_MERGE_SPLITS ? max_splits : MAX_MERGE_SPLITS)) pps *= 2;
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

}  // namespace fkv
