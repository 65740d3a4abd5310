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
  uint32_t red_n[kWaves];
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

// Returns the k-th largest value (1 <= k <= number of values incl. -inf entries); -inf when
// fewer than k values are finite.  All 256 threads must call it; result in every thread.
template <int NVAL>
__device__ float topk_threshold(const float (&x)[NVAL], int k, TopkSmem& ts) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  // range and count of the finite values
  float lo = INFINITY, hi = -INFINITY;
  uint32_t n = 0;
#pragma unroll
  for (int i = 0; i < NVAL; ++i) {
    const bool fin = x[i] > -INFINITY;
    lo = fin ? fminf(lo, x[i]) : lo;
    hi = fmaxf(hi, x[i]);
    n += fin ? 1u : 0u;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    lo = fminf(lo, __shfl_xor(lo, o, 64));
    hi = fmaxf(hi, __shfl_xor(hi, o, 64));
    n += __shfl_xor(n, o, 64);
  }
  __syncthreads();
  if (lane == 0) { ts.red_lo[wv] = lo; ts.red_hi[wv] = hi; ts.red_n[wv] = n; }
  __syncthreads();
  lo = fminf(fminf(ts.red_lo[0], ts.red_lo[1]), fminf(ts.red_lo[2], ts.red_lo[3]));
  hi = fmaxf(fmaxf(ts.red_hi[0], ts.red_hi[1]), fmaxf(ts.red_hi[2], ts.red_hi[3]));
  n = ts.red_n[0] + ts.red_n[1] + ts.red_n[2] + ts.red_n[3];
  if ((uint32_t)k > n) return -INFINITY;
  uint32_t kk = (uint32_t)k;

  for (int iter = 0; iter < 12; ++iter) {
    if (!(hi > lo)) return hi;                       // every remaining candidate ties
    const float scale = (float)kBuckets / __fsub_rn(hi, lo);
    for (int i = tid; i < kBuckets; i += kThreads) ts.hist[i] = 0u;
    if (tid == 0) { ts.n_list = 0u; ts.key_min = 0xffffffffu; ts.key_max = 0u; }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NVAL; ++i)
      if (x[i] >= lo && x[i] <= hi) atomicAdd(&ts.hist[bucket_of(x[i], hi, scale)], 1u);
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
    if (nb <= (uint32_t)kListCap) {
#pragma unroll
      for (int i = 0; i < NVAL; ++i)
        if (x[i] >= lo && x[i] <= hi && bucket_of(x[i], hi, scale) == bsel) ts.list[atomicAdd(&ts.n_list, 1u)] = x[i];
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
      if (x[i] >= lo && x[i] <= hi && bucket_of(x[i], hi, scale) == bsel) {
        atomicMin(&ts.key_min, order_key(x[i]));
        atomicMax(&ts.key_max, order_key(x[i]));
      }
    __syncthreads();
    lo = key_value(ts.key_min);
    hi = key_value(ts.key_max);
    __syncthreads();
  }
  return hi;   // not reached for fp32 inputs: every step splits distinct values
}

}  // namespace csd
