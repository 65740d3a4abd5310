// Block-wide exact selection of the k-th largest value of a row held in registers (fp32,
// NVAL values per thread, TPB threads).  Used for the top-k truncation "keep l >= k-th
// largest", ties at the threshold all kept.
//
// Method: value-bucket refinement.  The finite values lie in [lo, hi].  2048 equal-width
// buckets over that range are counted with LDS atomics; the bucket that holds the k-th largest
// is found by a prefix sum; if it holds at most kListCap values (the "bracket") they are copied to
// LDS and the answer is found by counting ranks, otherwise the range is narrowed to that bucket's own
// minimum and maximum and the step repeats.  The bucket index is a monotone function of the
// value, so every value of a lower-numbered bucket is >= every value of a higher one.  For
// Gaussian-like logits one step leaves about ten candidates.
//
// The common case (no -inf entry in the row, one step) is kept short: the histogram pass is
// then three instructions and one LDS atomic per value, with no range test.
#pragma once
#include "device_utils.h"

namespace csd {

constexpr int kBuckets = 2048;
constexpr int kListCap = 1024;

template <int TPB> struct TopkSmem {
  uint32_t hist[kBuckets];
  float list[kListCap];
  float red_lo[TPB / 64], red_hi[TPB / 64];
  uint32_t wave_tot[TPB / 64];
  uint32_t n_list;
  uint32_t key_min, key_max;
  int bsel;
  uint32_t k_in_bucket, n_in_bucket;
  uint32_t n_keep;
  float thr;
};

// order-preserving map fp32 -> uint32 and back
__device__ __forceinline__ uint32_t order_key(float v) {
  uint32_t u = __float_as_uint(v);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// Bucket of a value v in [lo, hi]: scale = fl(kBucketSpan / (hi - lo)) makes the product stay
// below kBuckets (2047.99 (1 + 2^-24)^2 < 2048), so no clamp is needed; subtraction,
// multiplication and truncation are monotone, which is all the method relies on.
constexpr float kBucketSpan = 2047.99f;
__device__ __forceinline__ int bucket_of(float v, float hi, float scale) {
  return (int)__fmul_rn(__fsub_rn(hi, v), scale);
}

__device__ __forceinline__ float wave_min(float v) {
  v = fminf(v, dpp_f<kDppSwap1>(v));
  v = fminf(v, dpp_f<kDppSwap2>(v));
  v = fminf(v, dpp_f<kDppHalfMirror>(v));
  v = fminf(v, dpp_f<kDppMirror>(v));
  return fminf(fminf(lane_f(v, 0), lane_f(v, 16)), fminf(lane_f(v, 32), lane_f(v, 48)));
}

// Where the k-th largest value lies once the bucket steps have narrowed it down: either the value
// itself (exact: every remaining candidate ties, or fewer than k values are finite), or one
// bucket of at most kListCap values.  bucket_of(v, hi, scale) == bsel names the candidates, which
// all lie in [g_lo, g_hi]; values above g_hi are larger than every candidate, values below g_lo
// smaller; kk is the rank of the wanted value among the nb candidates.
struct TopkBracket {
  bool exact;
  float thr;                   // exact only
  float g_lo, g_hi, hi, scale;
  int bsel;
  uint32_t kk, nb;
};

// Bracket of the kk-th largest of the values of all threads that lie in [lo, hi]; the caller
// guarantees that lo and hi are the minimum and maximum of the finite values and that the LDS
// histogram is zero.  in_range: every value of every thread lies in [lo, hi] (no -inf entries), so
// the first pass needs no range test.  All TPB threads must call it; result in every thread, and
// the candidate list of the shared state is empty.
template <int NVAL, int TPB>
__device__ __forceinline__ TopkBracket kth_bracket(const uint32_t (&xw)[NVAL], uint32_t kk, float lo, float hi,
                                                   bool in_range, TopkSmem<TPB>& ts) {
  constexpr int kW = TPB / 64;            // waves
  constexpr int kPer = kBuckets / TPB;    // buckets owned by one thread in the prefix step
  auto X = [&](int i) { return __uint_as_float(xw[i]); };
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  TopkBracket br{true, hi, 0.f, 0.f, hi, 0.f, 0, kk, 0u};
  for (int iter = 0; iter < 16; ++iter) {
    br.thr = hi;
    if (!(hi > lo)) return br;                           // every remaining candidate ties
    const float width = __fsub_rn(hi, lo);
    const float scale = kBucketSpan / width;
    if (iter > 0) {       // the first pass finds the histogram zeroed by topk_prepare
      __syncthreads();
      for (int i = tid; i < kBuckets; i += TPB) ts.hist[i] = 0u;
      if (tid == 0) { ts.n_list = 0u; ts.key_min = 0xffffffffu; ts.key_max = 0u; }
      __syncthreads();
    }
    if (in_range) {
#pragma unroll
      for (int i = 0; i < NVAL; ++i) atomicAdd(&ts.hist[bucket_of(X(i), hi, scale)], 1u);
    } else {
#pragma unroll
      for (int i = 0; i < NVAL; ++i)
        if (X(i) >= lo && X(i) <= hi) atomicAdd(&ts.hist[bucket_of(X(i), hi, scale)], 1u);
    }
    __syncthreads();
    // bucket that holds the kk-th largest: thread t owns buckets [kPer t, kPer (t+1))
    uint32_t h[kPer], local = 0;
#pragma unroll
    for (int j = 0; j < kPer; ++j) { h[j] = ts.hist[tid * kPer + j]; local += h[j]; }
    const uint32_t incl = wave_scan_incl_u32(local);
    if (lane == 63) ts.wave_tot[wv] = incl;
    __syncthreads();
    uint32_t before = incl - local, total = 0;
#pragma unroll
    for (int w = 0; w < kW; ++w) {
      before += (w < wv) ? ts.wave_tot[w] : 0u;
      total += ts.wave_tot[w];
    }
    if (kk > total) { br.thr = -INFINITY; return br; }
    if (before < kk && kk <= before + local) {
      uint32_t cum = before;
#pragma unroll
      for (int j = 0; j < kPer; ++j) {
        if (cum < kk && kk <= cum + h[j]) { ts.bsel = tid * kPer + j; ts.k_in_bucket = kk - cum; ts.n_in_bucket = h[j]; }
        cum += h[j];
      }
    }
    __syncthreads();
    const int bsel = ts.bsel;
    const uint32_t nb = ts.n_in_bucket;
    kk = ts.k_in_bucket;
    // value interval that certainly contains bucket bsel (bucket edges +- 1e-5 of the range,
    // far more than the rounding of bucket_of) and lies inside [lo, hi]; exact membership is
    // re-checked on the few hits
    const float step = width * (1.0f / kBucketSpan);
    const float margin = width * 1e-5f;
    const float g_hi = fminf(hi, hi - (float)bsel * step + margin);
    const float g_lo = fmaxf(lo, hi - (float)(bsel + 1) * step - margin);
    if (nb <= (uint32_t)kListCap) {
      br.exact = false;
      br.g_lo = g_lo; br.g_hi = g_hi; br.hi = hi; br.scale = scale; br.bsel = bsel; br.kk = kk; br.nb = nb;
      return br;
    }
    // too many candidates (heavy ties or a very uneven row): narrow the range to this bucket
#pragma unroll
    for (int i = 0; i < NVAL; ++i)
      if (X(i) >= g_lo && X(i) <= g_hi) {
        if (bucket_of(X(i), hi, scale) == bsel) {
          // the empty asm pins the key computation to this rare path: the values do not change
          // between steps, and hoisting 'order_key' of all of them out of the step loop would
          // cost one register per value on the common path
          float xv = X(i);
          asm volatile("" : "+v"(xv));
          atomicMin(&ts.key_min, order_key(xv));
          atomicMax(&ts.key_max, order_key(xv));
        }
      }
    __syncthreads();
    lo = key_value(ts.key_min);
    hi = key_value(ts.key_max);
    in_range = false;
  }
  br.thr = hi;   // not reached for fp32 inputs: every step splits distinct values
  return br;
}

// The wanted value from its bracket: the candidates are copied to LDS and ranked.  All TPB threads
// must call it; result in every thread.
template <int NVAL, int TPB>
__device__ __forceinline__ float kth_from_bracket(const uint32_t (&xw)[NVAL], const TopkBracket& br, TopkSmem<TPB>& ts) {
  if (br.exact) return br.thr;
  auto X = [&](int i) { return __uint_as_float(xw[i]); };
  const int tid = threadIdx.x;
#pragma unroll
  for (int i = 0; i < NVAL; ++i)
    if (X(i) >= br.g_lo && X(i) <= br.g_hi) {
      if (bucket_of(X(i), br.hi, br.scale) == br.bsel) ts.list[atomicAdd(&ts.n_list, 1u)] = X(i);
    }
  __syncthreads();
  // the kk-th largest v has fewer than kk values above it and at least kk values >= it
  for (uint32_t i = tid; i < br.nb; i += TPB) {
    const float v = ts.list[i];
    uint32_t g = 0, ge = 0;
    for (uint32_t j = 0; j < br.nb; ++j) { g += ts.list[j] > v; ge += ts.list[j] >= v; }
    if (g < br.kk && br.kk <= ge) ts.thr = v;
  }
  __syncthreads();
  return ts.thr;
}

// Bracket of the k-th largest of all NVAL x TPB values (1 <= k <= their number, -inf entries
// included); exactly -inf when fewer than k values are finite.  row_max receives the largest value
// (-inf for a row without a finite entry).  All TPB threads must call it.
template <int NVAL, int TPB>
__device__ __forceinline__ TopkBracket topk_bracket(const uint32_t (&xw)[NVAL], int k, TopkSmem<TPB>& ts, float& row_max) {
  const TopkBracket none{true, -INFINITY, 0.f, 0.f, 0.f, 0.f, 0, 0u, 0u};
  auto X = [&](int i) { return __uint_as_float(xw[i]); };
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  float hi = X(0), lo = X(0);
#pragma unroll
  for (int i = 1; i < NVAL; ++i) {
    hi = fmaxf(hi, X(i));
    lo = fminf(lo, X(i));
  }
  lo = wave_min(lo);
  hi = wave_max(hi);
  if (lane == 0) { ts.red_lo[wv] = lo; ts.red_hi[wv] = hi; }
  __syncthreads();
  lo = ts.red_lo[0];
  hi = ts.red_hi[0];
#pragma unroll
  for (int w = 1; w < TPB / 64; ++w) { lo = fminf(lo, ts.red_lo[w]); hi = fmaxf(hi, ts.red_hi[w]); }
  row_max = hi;
  if (!(hi > -INFINITY)) return none;                // no finite value at all
  bool in_range = true;
  if (!(lo > -INFINITY)) {
    // the row has -inf entries (excluded tokens, or elements beyond V): the minimum of the
    // finite values is needed for the bucket range
    in_range = false;
    lo = INFINITY;
#pragma unroll
    for (int i = 0; i < NVAL; ++i) lo = (X(i) > -INFINITY) ? fminf(lo, X(i)) : lo;
    lo = wave_min(lo);
    __syncthreads();                                   // red_lo was read above
    if (lane == 0) ts.red_lo[wv] = lo;
    __syncthreads();
    lo = ts.red_lo[0];
#pragma unroll
    for (int w = 1; w < TPB / 64; ++w) lo = fminf(lo, ts.red_lo[w]);
  }
  return kth_bracket<NVAL, TPB>(xw, (uint32_t)k, lo, hi, in_range, ts);
}

// The k-th largest itself.
template <int NVAL, int TPB>
__device__ __forceinline__ float topk_threshold(const uint32_t (&xw)[NVAL], int k, TopkSmem<TPB>& ts, float& row_max) {
  const TopkBracket br = topk_bracket<NVAL, TPB>(xw, k, ts, row_max);
  return kth_from_bracket<NVAL, TPB>(xw, br, ts);
}

// Zero the histogram; call it (all threads) before topk_threshold, e.g. while loads are in flight.
template <int TPB> __device__ __forceinline__ void topk_prepare(TopkSmem<TPB>& ts) {
  for (int i = threadIdx.x; i < kBuckets; i += TPB) ts.hist[i] = 0u;
  if (threadIdx.x == 0) { ts.n_list = 0u; ts.key_min = 0xffffffffu; ts.key_max = 0u; }
}

}  // namespace csd
