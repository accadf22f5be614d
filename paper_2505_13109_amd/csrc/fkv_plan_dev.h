// Device code of the recall plan of one KV head (Sec. 4.1: the selected pages the GPU already holds are
// not transferred again): which pages of the new selection the page cache holds, and which slots the
// others go to.
// A page hits iff it is in the ACTIVE selection (it keeps that slot).  Misses go, in ascending page
// order, to the lowest-numbered slots the ACTIVE selection does not use; pool of 2k slots per head.
// Run by a whole block of NT threads (a multiple of 64); the ordered parts are done by its first wave.
#pragma once
#include "fkv_device.h"

namespace fkv {

constexpr int PLAN_MISS_BIT = 0x40000000;     // in the LDS copy of the new slots: the position was a miss

__host__ __device__ constexpr size_t plan_lds_ints(int k) { return (size_t)8 * k + 4; }

// The pointers are the head's own rows: new_ids, act_ids, act_slots, new_slots [k]; mh [1 + 3k] = count,
// then per miss its page id, its slot, its position in the picked list.
// sm: plan_lds_ints(k) ints of LDS.  ids_in_lds: sm's `nid` row (sm + 4k) already holds the new ids, all of
// them full pages or -1; else they are read from new_ids, and an id that is not a full page of the context
// (a caller's list may hold anything) is dropped: rewritten to -1 in new_ids, so that neither the gather nor
// attention ever forms its address.
// On return (after a barrier) sm + 5k holds the new slots, PLAN_MISS_BIT set where the page has to be fetched.
template <int NT>
__device__ __forceinline__ void plan_head(int32_t* new_ids, const int32_t* act_ids, const int32_t* act_slots,
                                          int32_t* new_slots, int32_t* mh, int k, int n_full, int32_t* sm,
                                          bool ids_in_lds) {
  int32_t* used = sm;                      // [2k]
  int32_t* aid = sm + 2 * k;               // [k]
  int32_t* aslot = aid + k;                // [k]
  int32_t* nid = aslot + k;                // [k]
  int32_t* nslot = nid + k;                // [k]
  int32_t* freelist = nslot + k;           // [2k]
  int32_t* n_act_sh = freelist + 2 * k;    // [1]
  const int tid = threadIdx.x, lane = tid & 63;
  for (int s = tid; s < 2 * k; s += NT) used[s] = 0;
  for (int i = tid; i < k; i += NT) {      // all lists in one round trip
    aid[i] = act_ids[i];
    aslot[i] = act_slots[i];
    if (!ids_in_lds) {
      const int32_t id = new_ids[i];
      nid[i] = id < n_full ? id : -1;
      if (id >= n_full) new_ids[i] = -1;
    }
  }
  __syncthreads();
  for (int i = tid; i < k; i += NT)
    if (aid[i] >= 0) used[aslot[i]] = 1;
  if (tid < 64) {
    int n = 0;
    for (int i = lane; i < k; i += 64) n += aid[i] >= 0 ? 1 : 0;
    n = (int)wave_sum_u32((uint32_t)n);    // ids are ascending, -1 padded at the end
    if (lane == 0) *n_act_sh = n;
  }
  __syncthreads();
  const int n_act = *n_act_sh;
  // hit or miss per picked page (binary search in the ACTIVE ids)
  for (int i = tid; i < k; i += NT) {
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
  if (tid < 64) {
    int base = 0;
    for (int s0 = 0; s0 < 2 * k; s0 += 64) {
      const int s = s0 + lane;
      const uint32_t f = (s < 2 * k && !used[s]) ? 1u : 0u;
      const uint32_t incl = wave_scan_u32(f);
      if (f) freelist[base + (int)incl - 1] = s;
      base += (int)__builtin_amdgcn_readlane((int)incl, 63);
    }
  }
  __syncthreads();
  // the r-th miss (ascending page id) takes the r-th free slot
  if (tid < 64) {
    int n_miss = 0;
    for (int i0 = 0; i0 < k; i0 += 64) {
      const int i = i0 + lane;
      const uint32_t f = (i < k && nslot[i] == -2) ? 1u : 0u;
      const uint32_t incl = wave_scan_u32(f);
      if (f) {
        const int r = n_miss + (int)incl - 1;
        const int s = freelist[r];
        nslot[i] = s | PLAN_MISS_BIT;
        mh[1 + r] = nid[i];
        mh[1 + k + r] = s;
        mh[1 + 2 * k + r] = i;
      }
      n_miss += (int)__builtin_amdgcn_readlane((int)incl, 63);
    }
    if (lane == 0) mh[0] = n_miss;
  }
  __syncthreads();
  for (int i = tid; i < k; i += NT) {
    const int s = nslot[i];
    new_slots[i] = s < 0 ? s : (s & ~PLAN_MISS_BIT);
  }
}

}  // namespace fkv
