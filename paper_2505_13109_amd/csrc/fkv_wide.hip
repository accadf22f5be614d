// The selection of one KV head spread over several blocks, for long candidate lists (Sec. 3.2: softmax over
// the candidate pages, mean over the group, top-k).  One block per head is a chain of block-wide passes over
// all n candidates (18 us for 4K candidates); here the candidates are cut into B slices and the passes that
// need a value of the whole head are separated by launches instead:
//   scoring launch   every scoring block leaves the per-head maxima of the weights it wrote (a maximum is exact
//                    and has no order);
//   wide_z_kernel    block (slice, head): the head's maxima from those, the fixed-point softmax numerators of
//                    its slice, their integer sum added to the head's Z (64-bit integer atomic: exact, no order);
//   wide_pick_kernel block (slice, head): pooled scores of its slice, the slice's own top-k (any page of the
//                    head's top-k is in its slice's top-k under the same order), written out ascending by page;
//                    the block that finishes a head last merges the B short lists -- they are ascending by page
//                    id as a whole, so the same radix select with "ties to the lower position" applies.
// The arithmetic is the one of the single-block selection (fkv_step_dev.h), value for value.
#include "fkv_step_dev.h"

#pragma clang fp contract(off)

namespace fkv {

struct WideArgs {
  int n_q, n_kv, k, max_pages;
  Geom g;
  int sel_pool;                 // FKV_POOL_MEAN_S or FKV_POOL_MAX_S
  const float* P;               // [heads * G][max_pages]
  float* score;                 // [heads][max_pages]
  int32_t* ids;                 // [heads][k]
  int32_t* ids_user;            // may be null
  const float* bmax;            // [heads][bmax_stride][MAX_G]: maxima left by the scoring blocks
  int bmax_stride, n_score_blocks;   // scoring blocks per head
  float* hmax;                  // [heads][MAX_G]: the head's maxima (written by slice 0 of wide_z_kernel)
  unsigned long long* zsum;     // [heads][MAX_G]
  uint32_t* cand_key;           // [heads][B][k]
  int32_t* cand_id;             // [heads][B][k]
  int* counters;                // [heads]
  int B, slice;                 // slices per head, candidates per slice (the last one may be shorter)
};

template <int G>
__global__ __launch_bounds__(STEP_THREADS) void wide_z_kernel(WideArgs a) {
  __shared__ unsigned long long s_redz[STEP_WAVES][G];
  const int s = blockIdx.x, head = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = head / a.n_kv, m = head % a.n_kv;
  const int j_lo = s * a.slice, j_hi = min(a.g.n_cand, j_lo + a.slice);
  const float* Pm = a.P + (size_t)(b * a.n_q + m * G) * a.max_pages + a.g.cand_lo;
  // the head's maxima: over the scoring blocks' maxima
  __shared__ float s_mx[STEP_WAVES][G];
  float mx[G];
#pragma unroll
  for (int gg = 0; gg < G; ++gg) mx[gg] = -__builtin_inff();
  for (int blk = tid; blk < a.n_score_blocks; blk += STEP_THREADS) {
#pragma unroll
    for (int gg = 0; gg < G; ++gg) mx[gg] = fmaxf(mx[gg], a.bmax[((size_t)head * a.bmax_stride + blk) * MAX_G + gg]);
  }
#pragma unroll
  for (int gg = 0; gg < G; ++gg) {
    const float w = wave_max_f32(mx[gg]);
    if (lane == 0) s_mx[wave][gg] = w;
  }
  __syncthreads();
#pragma unroll
  for (int gg = 0; gg < G; ++gg) {
    float v = s_mx[0][gg];
#pragma unroll
    for (int w = 1; w < STEP_WAVES; ++w) v = fmaxf(v, s_mx[w][gg]);
    mx[gg] = v;
  }
  if (s == 0 && tid < G) a.hmax[(size_t)head * MAX_G + tid] = mx[tid];
  unsigned long long z[G];
#pragma unroll
  for (int gg = 0; gg < G; ++gg) z[gg] = 0;
  for (int j = j_lo + tid; j < j_hi; j += STEP_THREADS) {
#pragma unroll
    for (int gg = 0; gg < G; ++gg) z[gg] += softmax_fixed(Pm[(size_t)gg * a.max_pages + j], mx[gg]);
  }
#pragma unroll
  for (int gg = 0; gg < G; ++gg) {
    const unsigned long long w = wave_sum_u48(z[gg]);     // < 2^31 * ceil(slice / threads)
    if (lane == 0) s_redz[wave][gg] = w;
  }
  __syncthreads();
  if (tid < G) {
    unsigned long long v = 0;
#pragma unroll
    for (int w = 0; w < STEP_WAVES; ++w) v += s_redz[w][tid];
    atomicAdd(a.zsum + (size_t)head * MAX_G + tid, v);
  }
}

template <int G>
__global__ __launch_bounds__(STEP_THREADS) void wide_pick_kernel(WideArgs a) {
  extern __shared__ uint32_t dyn[];                        // keys: max(slice, B * k) entries, then B * k page ids
  __shared__ uint32_t hist[4][256];
  __shared__ uint32_t s_scan[STEP_WAVES];
  const int s = blockIdx.x, head = blockIdx.y, tid = threadIdx.x;
  const int b = head / a.n_kv, m = head % a.n_kv;
  const int n = a.g.n_cand, k = a.k, kk = a.g.k_eff;
  const int j_lo = s * a.slice, n_s = min(n, j_lo + a.slice) - j_lo;
  const float* Pm = a.P + (size_t)(b * a.n_q + m * G) * a.max_pages + a.g.cand_lo + j_lo;
  uint32_t* key = dyn;
  float mx[G];
  double zd[G], zr[G];
#pragma unroll
  for (int gg = 0; gg < G; ++gg) {
    mx[gg] = a.hmax[(size_t)head * MAX_G + gg];
    zd[gg] = (double)a.zsum[(size_t)head * MAX_G + gg];
    zr[gg] = reciprocal_near(zd[gg]);
  }
#pragma unroll
  for (int p = 0; p < 4; ++p)
    if (tid < 256) hist[p][tid] = 0;
  __syncthreads();
  for (int j = tid; j < n_s; j += STEP_THREADS) {
    uint32_t e[G];
#pragma unroll
    for (int gg = 0; gg < G; ++gg) e[gg] = softmax_fixed(Pm[(size_t)gg * a.max_pages + j], mx[gg]);
    const float sc = pooled_score<G>(e, zd, zr, a.sel_pool);
    a.score[(size_t)head * a.max_pages + a.g.cand_lo + j_lo + j] = sc;
    const uint32_t kj = score_key(sc);
    key[j] = kj;
    atomicAdd(&hist[3][kj >> 24], 1u);
  }
  __syncthreads();
  // the slice's own top-k, ascending by page, for the merge
  const int kk_s = min(kk, n_s);
  uint32_t* ck = a.cand_key + ((size_t)head * a.B + s) * k;
  int32_t* ci = a.cand_id + ((size_t)head * a.B + s) * k;
  if (kk_s > 0)
    radix_topk(key, n_s, kk_s, hist, s_scan, [&](int pos, int j) {
      __hip_atomic_store(ck + pos, key[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(ci + pos, a.g.cand_lo + j_lo + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    });
  if (!last_block_done(a.counters + head, a.B)) return;

  // ---- merge of the B short lists by the block that finished the head last ----
  int32_t* out = a.ids + (size_t)head * k;
  int32_t* outu = a.ids_user ? a.ids_user + (size_t)head * k : nullptr;
  uint32_t* mkey = dyn;
  int32_t* mid = reinterpret_cast<int32_t*>(dyn + max(a.slice, a.B * k));
#pragma unroll
  for (int p = 0; p < 4; ++p)
    if (tid < 256) hist[p][tid] = 0;
  __syncthreads();                                         // (also: every thread is done with the slice's keys)
  int n_m = 0;                                             // merged length; list s2 starts at n_m
  for (int s2 = 0; s2 < a.B; ++s2) {
    const int len = max(0, min(kk, min(n, (s2 + 1) * a.slice) - s2 * a.slice));
    const uint32_t* ck2 = a.cand_key + ((size_t)head * a.B + s2) * k;
    const int32_t* ci2 = a.cand_id + ((size_t)head * a.B + s2) * k;
    for (int i = tid; i < len; i += STEP_THREADS) {
      const uint32_t kj = __hip_atomic_load(ck2 + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      mkey[n_m + i] = kj;
      mid[n_m + i] = __hip_atomic_load(ci2 + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      atomicAdd(&hist[3][kj >> 24], 1u);
    }
    n_m += len;
  }
  __syncthreads();
  radix_topk(mkey, n_m, kk, hist, s_scan, [&](int pos, int p) {
    out[pos] = mid[p];
    if (outu) outu[pos] = mid[p];
  });
  for (int i = kk + tid; i < k; i += STEP_THREADS) {       // padding
    out[i] = -1;
    if (outu) outu[i] = -1;
  }
  if (tid < MAX_G) a.zsum[(size_t)head * MAX_G + tid] = 0;   // clean slate for the next step's sums
}

// slices of about one candidate per thread; false if this shape keeps the single-block selection
bool wide_plan(const Dims& d, const Geom& g, int* B, int* slice) {
  // Candidates per head from which the spread pays.  Its three launches are a chain of dependent round trips
  // of their own (maxima -> sums -> short lists -> counter -> merge): measured on one head's list, scan
  // included, 23.5 us against 22.8 us for the single block at 4064 candidates, 32.0 against 43.4 at 8160,
  // 38.8 against 73.6 at 15.3K.
  constexpr int kWideFrom = 5120;
  if (d.sel_pool > 1 || g.n_cand < kWideFrom || g.k_eff < 1) return false;
  int nb = (g.n_cand + STEP_THREADS - 1) / STEP_THREADS;
  if (nb > WIDE_MAX_SLICES) nb = WIDE_MAX_SLICES;
  if ((long)nb * d.k > 4096) return false;  // the merged list has to fit the last block's LDS comfortably
  *B = nb;
  *slice = (g.n_cand + nb - 1) / nb;
  return true;
}

template <int G>
static void launch_wide_g(const WideArgs& a, int heads, hipStream_t st) {
  const size_t lds = ((size_t)max(a.slice, a.B * a.k) + (size_t)a.B * a.k) * sizeof(uint32_t);
  dim3 grid(a.B, heads);
  wide_z_kernel<G><<<grid, STEP_THREADS, 0, st>>>(a);
  wide_pick_kernel<G><<<grid, STEP_THREADS, lds, st>>>(a);
}

void launch_wide_select(const Dims& d, const StepIO& io, Geom g, int B, int slice, int n_score_blocks, hipStream_t st) {
  WideArgs a{};
  a.n_q = d.n_q; a.n_kv = d.n_kv; a.k = d.k; a.max_pages = d.max_pages; a.g = g; a.sel_pool = d.sel_pool;
  a.P = io.P; a.score = io.score; a.ids = io.ids; a.ids_user = io.ids_user;
  a.bmax = io.bmax; a.bmax_stride = io.bmax_stride; a.n_score_blocks = n_score_blocks;
  a.hmax = io.hmax; a.zsum = io.zsum; a.cand_key = io.cand_key; a.cand_id = io.cand_id; a.counters = io.wide_counters;
  a.B = B; a.slice = slice;
  const int heads = d.batch * d.n_kv;
  switch (d.G) {
#define FKV_CASE(GG) case GG: launch_wide_g<GG>(a, heads, st); break;
    FKV_CASE(1) FKV_CASE(2) FKV_CASE(3) FKV_CASE(4) FKV_CASE(5) FKV_CASE(6) FKV_CASE(7) FKV_CASE(8)
#undef FKV_CASE
    default: break;
  }
}

}  // namespace fkv
