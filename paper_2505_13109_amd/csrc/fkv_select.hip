// Correction test, page weights, softmax -> group-mean pooling and top-k.
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
//   pooling: fl32( (sum_g fp64(E_g) / fp64(Z_g), g ascending) / fp64(G) );
//   top-k:   radix select on the fp32 bit pattern, ties to the lower page id.
#include "fkv_internal.h"

#pragma clang fp contract(off)

namespace fkv {

template <int DT> struct Unpack;
template <> struct Unpack<0> {   // fp16 pair in a 32-bit word
  static __device__ __forceinline__ float lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu)); }
  static __device__ __forceinline__ float hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }
};
template <> struct Unpack<1> {   // bf16 pair
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

// ---------------------------------------------------------------------------------
// Correction test (Sec. 3.1, 3.3).  grid (n_kv, batch), 128 threads = channels.
// ---------------------------------------------------------------------------------
template <int DT>
__global__ __launch_bounds__(128) void corr_kernel(const uint16_t* __restrict__ q,
                                                   const uint16_t* __restrict__ q_prev,
                                                   uint16_t* __restrict__ q_stage, int have_prev,
                                                   float tau, uint8_t* __restrict__ flags,
                                                   uint8_t* __restrict__ flags_user,
                                                   double* __restrict__ cosine, int n_q, int n_kv, int G) {
  __shared__ double red[3][128];
  __shared__ double cg[MAX_G];
  const int m = blockIdx.x, b = blockIdx.y, c = threadIdx.x;
  for (int g = 0; g < G; ++g) {
    const size_t idx = (size_t)(b * n_q + m * G + g) * D + c;
    const uint16_t qb = q[idx];
    double cosv = 0.0;
    if (have_prev) {
      const double a = (double)(DT == 0 ? Unpack<0>::lo(qb) : Unpack<1>::lo(qb));
      const uint16_t pb = q_prev[idx];
      const double p = (double)(DT == 0 ? Unpack<0>::lo(pb) : Unpack<1>::lo(pb));
      red[0][c] = a * p;
      red[1][c] = a * a;
      red[2][c] = p * p;
      __syncthreads();
      for (int s = 64; s > 0; s >>= 1) {
        if (c < s) {
          red[0][c] += red[0][c + s];
          red[1][c] += red[1][c + s];
          red[2][c] += red[2][c + s];
        }
        __syncthreads();
      }
      if (c == 0) {
        const double den = sqrt(red[1][0] * red[2][0]);
        cosv = den > 0.0 ? red[0][0] / den : 0.0;
        cg[g] = cosv;
        cosine[b * n_q + m * G + g] = cosv;
      }
      __syncthreads();
    } else if (c == 0) {
      cosine[b * n_q + m * G + g] = 0.0;
    }
    q_stage[idx] = qb;
  }
  if (c == 0) {
    uint8_t f = 1;
    if (have_prev) {
      double acc = 0.0;
      for (int g = 0; g < G; ++g) acc = acc + cg[g];
      f = (acc / (double)G) < (double)tau ? 1 : 0;
    }
    flags[b * n_kv + m] = f;
    if (flags_user) flags_user[b * n_kv + m] = f;
  }
}

// ---------------------------------------------------------------------------------
// Page weights P^h_j from the min-max summaries (Sec. 3.2).
// A 16-lane group owns one page: lane c8 holds channels 8*c8 .. 8*c8+7 of kmax and
// kmin (one 16-byte load each, 1 KiB contiguous per wave and array), so a wave
// scores 4 pages and a 256-thread block 16 pages per pass.
// grid (ceil(n_cand / (16*PASSES)), n_kv, batch).
// ---------------------------------------------------------------------------------
constexpr int SCORE_PASSES = 1;

template <int DT, int G>
__global__ __launch_bounds__(256) void score_kernel(const uint16_t* __restrict__ summ,
                                                    const uint16_t* __restrict__ q,
                                                    float* __restrict__ P, Geom g, int n_q, int n_kv,
                                                    int max_pages) {
  const int m = blockIdx.y, b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = lane >> 4, c8 = lane & 15;
  const uint16_t* kmax = summ + ((size_t)((b * n_kv + m) * 2 + 0) * max_pages) * D;
  const uint16_t* kmin = summ + ((size_t)((b * n_kv + m) * 2 + 1) * max_pages) * D;

  // summaries first: their addresses do not depend on q
  uint4 wmax[SCORE_PASSES], wmin[SCORE_PASSES];
  int page[SCORE_PASSES];
#pragma unroll
  for (int ps = 0; ps < SCORE_PASSES; ++ps) {
    const int j = (blockIdx.x * SCORE_PASSES + ps) * 16 + wave * 4 + grp;
    page[ps] = j < g.n_cand ? g.cand_lo + j : -1;
    const int jj = j < g.n_cand ? g.cand_lo + j : g.cand_lo;
    wmax[ps] = *reinterpret_cast<const uint4*>(kmax + (size_t)jj * D + c8 * 8);
    wmin[ps] = *reinterpret_cast<const uint4*>(kmin + (size_t)jj * D + c8 * 8);
  }
  // q split by sign: q+ multiplies kmax, q- multiplies kmin; one of the two products is zero
  float qp[G][8], qn[G][8];
#pragma unroll
  for (int gg = 0; gg < G; ++gg) {
    const uint4 w = *reinterpret_cast<const uint4*>(q + (size_t)(b * n_q + m * G + gg) * D + c8 * 8);
    float f[8];
    unpack8<DT>(w, f);
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      qp[gg][c] = f[c] >= 0.0f ? f[c] : 0.0f;
      qn[gg][c] = f[c] >= 0.0f ? 0.0f : f[c];
    }
  }
  const float scale = 0x1.6a09e6p-4f;   // fl32(1/sqrt(128))
#pragma unroll
  for (int ps = 0; ps < SCORE_PASSES; ++ps) {
    float kx[8], kn[8];
    unpack8<DT>(wmax[ps], kx);
    unpack8<DT>(wmin[ps], kn);
#pragma unroll
    for (int gg = 0; gg < G; ++gg) {
      // chunk sum, left to right; each fma adds one exact product (the other one is +-0)
      float s = 0.0f;
#pragma unroll
      for (int c = 0; c < 8; ++c) {
        s = __builtin_fmaf(qp[gg][c], kx[c], s);
        s = __builtin_fmaf(qn[gg][c], kn[c], s);
      }
      // adjacent-pair tree over the 16 chunk sums
      s = s + __shfl_xor(s, 1, 64);
      s = s + __shfl_xor(s, 2, 64);
      s = s + __shfl_xor(s, 4, 64);
      s = s + __shfl_xor(s, 8, 64);
      const float w = s * scale;
      if (c8 == gg && page[ps] >= 0) P[(size_t)(b * n_q + m * G + gg) * max_pages + page[ps]] = w;
    }
  }
}

// ---------------------------------------------------------------------------------
// softmax -> group mean -> top-k.  One 512-thread block per (KV head, request).
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
  float e = __builtin_ldexpf(r, (int)n);
  if (t < -64.0f) e = 0.0f;
  return (uint32_t)__builtin_rintf(e * 2147483648.0f);
}

constexpr int SEL_THREADS = 512;
constexpr int SEL_WAVES = SEL_THREADS / 64;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) v = fmaxf(v, __shfl_xor(v, s, 64));
  return v;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
  for (int s = 32; s > 0; s >>= 1) v += __shfl_xor(v, s, 64);
  return v;
}

__global__ __launch_bounds__(SEL_THREADS) void select_kernel(const float* __restrict__ P,
                                                             float* __restrict__ score_out,
                                                             int32_t* __restrict__ ids,
                                                             int32_t* __restrict__ ids_user, Geom g,
                                                             int n_q, int n_kv, int G, int k,
                                                             int max_pages) {
  extern __shared__ uint32_t key[];                 // n_cand pooled scores as ordered bit patterns
  __shared__ float s_max[MAX_G];
  __shared__ unsigned long long s_z[MAX_G];
  __shared__ float s_redf[SEL_WAVES];
  __shared__ unsigned long long s_redz[SEL_WAVES];
  __shared__ uint32_t hist[256];
  __shared__ uint32_t s_prefix, s_remaining;
  __shared__ uint32_t s_scan[SEL_WAVES];

  const int m = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int n = g.n_cand, lo = g.cand_lo, kk = g.k_eff;
  int32_t* out = ids + (size_t)(b * n_kv + m) * k;
  int32_t* outu = ids_user ? ids_user + (size_t)(b * n_kv + m) * k : nullptr;
  for (int i = kk + tid; i < k; i += SEL_THREADS) {
    out[i] = -1;
    if (outu) outu[i] = -1;
  }
  if (kk == 0) return;

  // per-head maximum over the candidates
  for (int gg = 0; gg < G; ++gg) {
    const float* Ph = P + (size_t)(b * n_q + m * G + gg) * max_pages + lo;
    float mx = -__builtin_inff();
    for (int j = tid; j < n; j += SEL_THREADS) mx = fmaxf(mx, Ph[j]);
    mx = wave_max(mx);
    if (lane == 0) s_redf[wave] = mx;
    __syncthreads();
    if (tid == 0) {
      float v = s_redf[0];
      for (int w = 1; w < SEL_WAVES; ++w) v = fmaxf(v, s_redf[w]);
      s_max[gg] = v;
    }
    __syncthreads();
  }
  // integer softmax denominators
  for (int gg = 0; gg < G; ++gg) {
    const float* Ph = P + (size_t)(b * n_q + m * G + gg) * max_pages + lo;
    const float mx = s_max[gg];
    unsigned long long z = 0;
    for (int j = tid; j < n; j += SEL_THREADS) z += softmax_fixed(Ph[j], mx);
    z = wave_sum_u64(z);
    if (lane == 0) s_redz[wave] = z;
    __syncthreads();
    if (tid == 0) {
      unsigned long long v = 0;
      for (int w = 0; w < SEL_WAVES; ++w) v += s_redz[w];
      s_z[gg] = v;
    }
    __syncthreads();
  }
  // pooled score of each candidate
  for (int j = tid; j < n; j += SEL_THREADS) {
    double acc = 0.0;
    for (int gg = 0; gg < G; ++gg) {
      const float p = P[(size_t)(b * n_q + m * G + gg) * max_pages + lo + j];
      acc = acc + (double)softmax_fixed(p, s_max[gg]) / (double)s_z[gg];
    }
    const float sc = (float)(acc / (double)G);
    key[j] = __float_as_uint(sc);                  // sc >= 0: bit patterns order like the values
    score_out[(size_t)(b * n_kv + m) * max_pages + lo + j] = sc;
  }
  if (tid == 0) { s_prefix = 0; s_remaining = (uint32_t)kk; }
  __syncthreads();

  // radix select: the kk-th largest key, one byte at a time from the top
  for (int pass = 3; pass >= 0; --pass) {
    for (int i = tid; i < 256; i += SEL_THREADS) hist[i] = 0;
    __syncthreads();
    const uint32_t prefix = s_prefix;
    const int shift = pass * 8;
    for (int j = tid; j < n; j += SEL_THREADS) {
      const uint32_t kj = key[j];
      if (pass == 3 || (kj >> (shift + 8)) == prefix) atomicAdd(&hist[(kj >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid == 0) {
      uint32_t rem = s_remaining;
      int bin = 255;
      while (hist[bin] < rem) { rem -= hist[bin]; --bin; }
      s_remaining = rem;                            // how many to take inside `bin`
      s_prefix = (prefix << 8) | (uint32_t)bin;
    }
    __syncthreads();
  }
  const uint32_t T = s_prefix;                       // the kk-th largest key
  const uint32_t take_eq = s_remaining;              // keys equal to T to take, lowest ids first

  // ordered compaction: thread t owns the contiguous ids [t*per, (t+1)*per)
  const int per = (n + SEL_THREADS - 1) / SEL_THREADS;
  const int j0 = tid * per, j1 = min(n, j0 + per);
  uint32_t cnt = 0;                                  // low 16 bits: keys > T, high 16 bits: keys == T
  for (int j = j0; j < j1; ++j) {
    const uint32_t kj = key[j];
    cnt += (kj > T ? 1u : 0u) + (kj == T ? 0x10000u : 0u);
  }
  uint32_t incl = cnt;
#pragma unroll
  for (int s = 1; s < 64; s <<= 1) {
    const uint32_t v = __shfl_up(incl, s, 64);
    if (lane >= s) incl += v;
  }
  if (lane == 63) s_scan[wave] = incl;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += s_scan[w];
  uint32_t excl = base + incl - cnt;
  uint32_t gt_before = excl & 0xffffu, eq_before = excl >> 16;
  for (int j = j0; j < j1; ++j) {
    const uint32_t kj = key[j];
    if (kj > T || (kj == T && eq_before < take_eq)) {
      const uint32_t pos = gt_before + min(eq_before, take_eq);
      out[pos] = lo + j;
      if (outu) outu[pos] = lo + j;
    }
    gt_before += (kj > T);
    eq_before += (kj == T);
  }
}

// ---- launch wrappers ----------------------------------------------------------------
void launch_corr(const Dims& d, const uint16_t* q, const uint16_t* q_prev, uint16_t* q_stage,
                 int have_prev, float tau, uint8_t* flags, uint8_t* flags_user, double* cosine,
                 hipStream_t st) {
  dim3 grid(d.n_kv, d.batch);
  if (d.dtype == 0) corr_kernel<0><<<grid, 128, 0, st>>>(q, q_prev, q_stage, have_prev, tau, flags, flags_user, cosine, d.n_q, d.n_kv, d.G);
  else              corr_kernel<1><<<grid, 128, 0, st>>>(q, q_prev, q_stage, have_prev, tau, flags, flags_user, cosine, d.n_q, d.n_kv, d.G);
}

template <int DT>
static void launch_score_dt(const Dims& d, const uint16_t* summ, const uint16_t* q, float* P, Geom g, hipStream_t st) {
  dim3 grid((g.n_cand + 16 * SCORE_PASSES - 1) / (16 * SCORE_PASSES), d.n_kv, d.batch);
  switch (d.G) {
#define FKV_CASE(GG) case GG: score_kernel<DT, GG><<<grid, 256, 0, st>>>(summ, q, P, g, d.n_q, d.n_kv, d.max_pages); break;
    FKV_CASE(1) FKV_CASE(2) FKV_CASE(3) FKV_CASE(4) FKV_CASE(5) FKV_CASE(6) FKV_CASE(7) FKV_CASE(8)
#undef FKV_CASE
    default: break;
  }
}

void launch_score(const Dims& d, const uint16_t* summ, const uint16_t* q, float* P, Geom g, hipStream_t st) {
  if (g.n_cand <= 0) return;
  if (d.dtype == 0) launch_score_dt<0>(d, summ, q, P, g, st);
  else              launch_score_dt<1>(d, summ, q, P, g, st);
}

void launch_select(const Dims& d, const float* P, float* score, int32_t* ids, int32_t* ids_user,
                   Geom g, hipStream_t st) {
  if (d.k == 0) return;
  dim3 grid(d.n_kv, d.batch);
  const size_t lds = (size_t)(g.n_cand > 0 ? g.n_cand : 1) * sizeof(uint32_t);
  select_kernel<<<grid, SEL_THREADS, lds, st>>>(P, score, ids, ids_user, g, d.n_q, d.n_kv, d.G, d.k, d.max_pages);
}

}  // namespace fkv
