// Device-side helpers shared by the kernel files.
#pragma once
#include "fkv_internal.h"

namespace fkv {

// one storage element / a packed pair of them -> fp32 (exact)
template <int DT> struct Unpack;
template <> struct Unpack<0> {   // fp16
  static __device__ __forceinline__ float one(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
  static __device__ __forceinline__ float lo(uint32_t w) { return one((uint16_t)(w & 0xffffu)); }
  static __device__ __forceinline__ float hi(uint32_t w) { return one((uint16_t)(w >> 16)); }
};
template <> struct Unpack<1> {   // bf16
  static __device__ __forceinline__ float one(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
  static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
  static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
};
template <int DT>
__device__ __forceinline__ void unpack8(const uint4& w, float* f) {
  f[0] = Unpack<DT>::lo(w.x); f[1] = Unpack<DT>::hi(w.x);
  f[2] = Unpack<DT>::lo(w.y); f[3] = Unpack<DT>::hi(w.y);
  f[4] = Unpack<DT>::lo(w.z); f[5] = Unpack<DT>::hi(w.z);
  f[6] = Unpack<DT>::lo(w.w); f[7] = Unpack<DT>::hi(w.w);
}

__device__ __forceinline__ int resident_unit(const PoolDesc& pd, int page) {
  if (pd.placement == 0) return page;
  return page < pd.ring_base ? page : pd.ring_base + page % pd.n_ring;
}
__device__ __forceinline__ size_t head_base(const PoolDesc& pd, int b, int m, int n_kv) {
  return (size_t)(b * n_kv + m) * pd.units_per_head;
}
__device__ __forceinline__ size_t summ_idx(int b, int m, int n_kv, int which, int max_pages, int page) {
  return ((size_t)((b * n_kv + m) * 2 + which) * max_pages + page) * D;
}

// correction flag of a KV head from the similarities of its G query heads (Sec. 3.3): the
// group-pooled similarity strictly below tau.  pool: 0 mean (sum in head order / G), 1 maximum,
// 2 minimum (App. B.3).  fp64, one thread.
__device__ __forceinline__ int pooled_flag(const double* c, int G, float tau, int pool) {
  double acc = c[0];
  for (int gg = 1; gg < G; ++gg) {
    const double v = c[gg];
    if (pool == 0) acc = acc + v;
    else if (pool == 1) acc = v > acc ? v : acc;
    else acc = v < acc ? v : acc;
  }
  if (pool == 0) acc = acc / (double)G;
  return acc < (double)tau ? 1 : 0;
}

// cosine of one query head against the previous step's query (Sec. 3.1); one wave, fp64
template <int DT>
__device__ __forceinline__ double head_cosine(const uint16_t* q, const uint16_t* q_prev, int lane, uint32_t* q_word) {
  const uint32_t qw = *reinterpret_cast<const uint32_t*>(q + lane * 2);
  const uint32_t pw = *reinterpret_cast<const uint32_t*>(q_prev + lane * 2);
  if (q_word) *q_word = qw;
  const double a0 = (double)Unpack<DT>::lo(qw), a1 = (double)Unpack<DT>::hi(qw);
  const double p0 = (double)Unpack<DT>::lo(pw), p1 = (double)Unpack<DT>::hi(pw);
  double dot = a0 * p0 + a1 * p1, na = a0 * a0 + a1 * a1, nb = p0 * p0 + p1 * p1;
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) {
    dot += __shfl_xor(dot, s, 64);
    na += __shfl_xor(na, s, 64);
    nb += __shfl_xor(nb, s, 64);
  }
  const double den = sqrt(na * nb);
  return den > 0.0 ? dot / den : 0.0;
}

// ---- wavefront reductions on the DPP cross-lane path (no LDS traffic) ------------------
// xor-1, xor-2 inside quads, then half-row and row mirrors: every lane of a 16-lane row ends
// with the row's result; two row broadcasts carry it on, lane 63 holds the wave's result.
template <typename OP>
__device__ __forceinline__ uint32_t wave_reduce_u32(uint32_t v, OP op) {
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, false));  // row_half_mirror
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, false));  // row_mirror
  // row_bcast:15 into rows 1 and 3, row_bcast:31 into rows 2 and 3; lanes not written keep v
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)OP::identity(), (int)v, 0x142, 0xa, 0xf, false));
  v = op(v, (uint32_t)__builtin_amdgcn_update_dpp((int)OP::identity(), (int)v, 0x143, 0xc, 0xf, false));
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}
struct OpMaxF32 {   // on bit patterns of floats
  static __device__ __forceinline__ uint32_t identity() { return 0xff800000u; }   // -inf
  __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const {
    return __float_as_uint(fmaxf(__uint_as_float(a), __uint_as_float(b)));
  }
};
struct OpAddU32 {
  static __device__ __forceinline__ uint32_t identity() { return 0u; }
  __device__ __forceinline__ uint32_t operator()(uint32_t a, uint32_t b) const { return a + b; }
};
__device__ __forceinline__ float wave_max_f32(float v) {
  return __uint_as_float(wave_reduce_u32(__float_as_uint(v), OpMaxF32()));
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) { return wave_reduce_u32(v, OpAddU32()); }
// sum of 64 values below 2^48 each, as two 24-bit-limb sums so that no 32-bit lane sum overflows
__device__ __forceinline__ unsigned long long wave_sum_u48(unsigned long long v) {
  const uint32_t l0 = (uint32_t)(v & 0xffffffu), l1 = (uint32_t)(v >> 24);
  return (unsigned long long)wave_sum_u32(l0) + ((unsigned long long)wave_sum_u32(l1) << 24);
}

// inclusive prefix sum across the 64 lanes (Hillis-Steele inside 16-lane rows, then two row broadcasts)
__device__ __forceinline__ uint32_t wave_scan_u32(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);   // row_shr:1, 0 shifted in
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);   // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);   // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);   // row_shr:8
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);  // rows 1,3 += total of rows 0,2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);  // rows 2,3 += total of lanes 0..31
  return v;
}

// ---- exchange between blocks of one launch ---------------------------------------
// Each XCD has its own L2, so data one block writes for another block of the same launch
// must not sit in (or be read from) a non-coherent L2 line.  A device-scope fence per
// block would write back and invalidate the whole L2 each time; instead the few values
// that are exchanged (page weights, attention partials) are written and read with
// relaxed device-scope atomics, which the hardware serves at the device coherence point.
__device__ __forceinline__ void st_dev(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev2(float* p, float a, float b) {   // p 8-byte aligned
  const unsigned long long w = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_dev2(const float* p) {
  const unsigned long long w = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                                 __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__uint_as_float((uint32_t)w), __uint_as_float((uint32_t)(w >> 32)));
}

// A picked page as one 32-bit value, for the exchange between the selecting block and waiting attention waves when the
// KV lives in a host pool: page id (< 2^16), page-cache slot (< 2^15), and whether the slot has yet to be filled from
// the host pool; all ones: no page at this position.
constexpr int TAGGED_MAX_PAGES = 1 << 16, TAGGED_MAX_SLOTS = 1 << 15;
__device__ __forceinline__ uint32_t tagged_pick(int id, int slot, bool miss) {
  return id < 0 ? 0xffffffffu : ((miss ? 0x80000000u : 0u) | ((uint32_t)slot << 16) | (uint32_t)id);
}
__device__ __forceinline__ void tagged_unpick(uint32_t w, int& id, int& slot, bool& miss) {
  if (w == 0xffffffffu) { id = -1; slot = -1; miss = false; return; }
  id = (int)(w & 0xffffu);
  slot = (int)((w >> 16) & 0x7fffu);
  miss = (w >> 31) != 0;
}

// All vector-memory operations this wave has issued so far -- loads and stores count on the same
// counter on this target -- have completed.  For a store issued at device scope (st_dev*: written
// through to the device coherence point) "completed" means it is visible to every compute unit of
// the GPU, which is what the release side of the exchange below needs; no L2 write-back is involved
// because nothing that is exchanged was written with a plain store.
__device__ __forceinline__ void wait_vector_memory() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// Release side of an exchange: every wave of the block waits for its own device-scope stores, the
// barrier then makes "all of the block's stores are visible" a fact thread 0 may publish.  The
// workgroup-scope fences only pin the compiler's ordering around the barrier.
__device__ __forceinline__ void block_release() {
  wait_vector_memory();
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __syncthreads();
}
// Acquire side: after thread 0 has observed the other blocks' publication, the barrier hands that
// knowledge to the block and the fence keeps every later (device-scope, ld_dev*) load behind it.
__device__ __forceinline__ void block_acquire() {
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// Block-wide "am I the last one?" for a group of `expected` blocks sharing `counter`.
// What the block stored with st_dev* before the call is visible device-wide when the counter is
// bumped (block_release), so the block that gets `true` can read every other block's values with
// ld_dev*.  Resets the counter for the next launch.
__device__ __forceinline__ bool last_block_done(int* counter, int expected) {
  __shared__ int s_last;
  block_release();
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (old == expected - 1);
    if (s_last) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  block_acquire();
  return s_last != 0;
}

}  // namespace fkv
