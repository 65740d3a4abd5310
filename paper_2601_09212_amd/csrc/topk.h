// Block-wide exact selection of the k-th largest value of a row held in registers (fp32,
// NT*kE values per thread, 256 threads).  Used for the top-k truncation "keep l >= k-th
// largest", ties at the threshold all kept.
//
// Method: value-bucket refinement.  The finite values lie in [lo, hi].  2048 equal-width
// buckets over that range are counted with LDS atomics; the bucket that holds the k-th largest
// is found by a prefix sum; if it holds at most kListCap values they are copied to LDS and the
// answer is found by counting ranks, otherwise the range is narrowed to that bucket's own
// minimum and maximum and the step repeats.  The bucket index is a monotone function of the
// value, so every value of a lower-numbered bucket is >= every value of a higher one.  For
// Gaussian-like logits one step leaves about ten candidates.
#pragma once
#include "device_utils.h"

namespace csd {

constexpr int kBuckets = 2048;
constexpr int kListCap = 1024;

struct TopkSmem {
  uint32_t hist[kBuckets];
  float list[kListCap];
  float red_lo[kWaves], red_hi[kWaves];
  uint32_t wave_tot[kWaves];
  uint32_t n_list;
  uint32_t key_min, key_max;
  int bsel;
  uint32_t k_in_bucket, n_in_bucket;
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

__device__ __forceinline__ int bucket_of(float v, float hi, float scale) {
  const int b = (int)__fmul_rn(__fsub_rn(hi, v), scale);
  return b > kBuckets - 1 ? kBuckets - 1 : b;
}

// k-th largest of the values of all threads that lie in [lo, hi]; the caller guarantees that lo
// and hi are the minimum and maximum of the finite values and that the LDS histogram is zero.
// Returns -inf when fewer than k values are finite.  All 256 threads must call it; result in
// every thread.
template <int NVAL>
__device__ __forceinline__ float kth_largest(const uint32_t (&xw)[NVAL], uint32_t kk, float lo, float hi,
                                             TopkSmem& ts) {
  constexpr bool exact_lo = true;
  auto X = [&](int i) { return __uint_as_float(xw[i]); };
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  bool narrowed = false;                               // hi is no longer the maximum of the values
  for (int iter = 0; iter < 16; ++iter) {
    if (!(hi > lo) && (exact_lo || narrowed)) return hi;   // every remaining candidate ties
    const float width = __fsub_rn(hi, lo);
    const float scale = (width > 0.f) ? (float)kBuckets / width : 0.f;
    if (iter > 0) {       // the first pass finds the histogram zeroed by topk_prepare
      __syncthreads();
      for (int i = tid; i < kBuckets; i += kThreads) ts.hist[i] = 0u;
      if (tid == 0) { ts.n_list = 0u; ts.key_min = 0xffffffffu; ts.key_max = 0u; }
      __syncthreads();
    }
    if (!narrowed) {
#pragma unroll
      for (int i = 0; i < NVAL; ++i)
        if (X(i) >= lo) atomicAdd(&ts.hist[bucket_of(X(i), hi, scale)], 1u);
    } else {
#pragma unroll
      for (int i = 0; i < NVAL; ++i)
        if (X(i) >= lo && X(i) <= hi) atomicAdd(&ts.hist[bucket_of(X(i), hi, scale)], 1u);
    }
    __syncthreads();
    // bucket that holds the kk-th largest: thread t owns buckets [8t, 8t+8)
    uint32_t h[8], local = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) { h[j] = ts.hist[tid * 8 + j]; local += h[j]; }
    uint32_t incl = local;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      uint32_t t = __shfl_up(incl, o, 64);
      if (lane >= o) incl += t;
    }
    if (lane == 63) ts.wave_tot[wv] = incl;
    __syncthreads();
    uint32_t before = incl - local;
    for (int w = 0; w < wv; ++w) before += ts.wave_tot[w];
    const uint32_t total = ts.wave_tot[0] + ts.wave_tot[1] + ts.wave_tot[2] + ts.wave_tot[3];
    if (kk > total) return (exact_lo || narrowed) ? -INFINITY : NAN;
    if (before < kk && kk <= before + local) {
      uint32_t cum = before;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (cum < kk && kk <= cum + h[j]) { ts.bsel = tid * 8 + j; ts.k_in_bucket = kk - cum; ts.n_in_bucket = h[j]; }
        cum += h[j];
      }
    }
    __syncthreads();
    const int bsel = ts.bsel;
    const uint32_t nb = ts.n_in_bucket;
    kk = ts.k_in_bucket;
    // value interval that certainly contains bucket bsel (bucket edges +- 1e-5 of the range,
    // far more than the rounding of bucket_of); exact membership is re-checked on the few hits
    const float step = width * (1.0f / kBuckets);
    const float margin = width * 1e-5f;
    const float g_hi = hi - (float)bsel * step + margin;
    const float g_lo = (bsel == kBuckets - 1 || !(width > 0.f)) ? lo : fmaxf(lo, hi - (float)(bsel + 1) * step - margin);
    if (nb <= (uint32_t)kListCap) {
#pragma unroll
      for (int i = 0; i < NVAL; ++i)
        if (X(i) >= g_lo && X(i) <= g_hi) {
          if (X(i) <= hi && bucket_of(X(i), hi, scale) == bsel) ts.list[atomicAdd(&ts.n_list, 1u)] = X(i);
        }
      __syncthreads();
      // the kk-th largest v has fewer than kk values above it and at least kk values >= it
      for (uint32_t i = tid; i < nb; i += kThreads) {
        const float v = ts.list[i];
        uint32_t g = 0, ge = 0;
        for (uint32_t j = 0; j < nb; ++j) { g += ts.list[j] > v; ge += ts.list[j] >= v; }
        if (g < kk && kk <= ge) ts.thr = v;
      }
      __syncthreads();
      return ts.thr;
    }
    // too many candidates (heavy ties or a very uneven row): narrow the range to this bucket
#pragma unroll
    for (int i = 0; i < NVAL; ++i)
      if (X(i) >= g_lo && X(i) <= g_hi) {
        if (X(i) <= hi && bucket_of(X(i), hi, scale) == bsel) {
          atomicMin(&ts.key_min, order_key(X(i)));
          atomicMax(&ts.key_max, order_key(X(i)));
        }
      }
    __syncthreads();
    lo = key_value(ts.key_min);
    hi = key_value(ts.key_max);
    narrowed = true;
  }
  return hi;   // not reached for fp32 inputs: every step splits distinct values
}

// Returns the k-th largest of all NVAL x 256 values (1 <= k <= their number, -inf entries
// included); -inf when fewer than k values are finite.  All 256 threads must call it.
template <int NVAL>
__device__ __forceinline__ float topk_threshold(const uint32_t (&xw)[NVAL], int k, TopkSmem& ts) {
  auto X = [&](int i) { return __uint_as_float(xw[i]); };
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  float hi = -INFINITY, lo = INFINITY;
#pragma unroll
  for (int i = 0; i < NVAL; ++i) {
    hi = fmaxf(hi, X(i));
    lo = (X(i) > -INFINITY) ? fminf(lo, X(i)) : lo;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    lo = fminf(lo, __shfl_xor(lo, o, 64));
    hi = fmaxf(hi, __shfl_xor(hi, o, 64));
  }
  if (lane == 0) { ts.red_lo[wv] = lo; ts.red_hi[wv] = hi; }
  __syncthreads();
  lo = fminf(fminf(ts.red_lo[0], ts.red_lo[1]), fminf(ts.red_lo[2], ts.red_lo[3]));
  hi = fmaxf(fmaxf(ts.red_hi[0], ts.red_hi[1]), fmaxf(ts.red_hi[2], ts.red_hi[3]));
  if (!(hi > -INFINITY)) return -INFINITY;           // no finite value at all
  return kth_largest<NVAL>(xw, (uint32_t)k, lo, hi, ts);
}

// Zero the histogram; call it (all threads) before topk_threshold, e.g. while loads are in flight.
__device__ __forceinline__ void topk_prepare(TopkSmem& ts) {
  for (int i = threadIdx.x; i < kBuckets; i += kThreads) ts.hist[i] = 0u;
  if (threadIdx.x == 0) { ts.n_list = 0u; ts.key_min = 0xffffffffu; ts.key_max = 0u; }
}

}  // namespace csd
