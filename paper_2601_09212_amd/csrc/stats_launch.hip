// Statistics pass of a verify / resample / diagnostics call: dispatch to the (dtype, transform)
// slices, and the one kernel of the pass that is not a template.
#include "stats_launch.h"

namespace csd {

// One workgroup per row: the digit of this radix pass that holds the k-th largest key.  Thread t
// owns the eight buckets 2047 - 8t .. 2040 - 8t, so that ascending thread order is descending key
// order.
__global__ __launch_bounds__(kThreads) void topk_radix_select_kernel(const KArgs a, int pass) {
  __shared__ uint32_t wave_tot[kWaves];
  const int r = blockIdx.x;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  uint32_t* hist = a.rk_hist + int64_t(r) * kRadixBuckets;
  const uint32_t k_rem = pass == 0 ? (uint32_t)a.top_k : a.rk_state[2 * r + 1];
  const uint32_t prefix = pass == 0 ? 0u : a.rk_state[2 * r];
  uint32_t h[8], local = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int bkt = kRadixBuckets - 1 - (threadIdx.x * 8 + j);
    h[j] = hist[bkt];
    hist[bkt] = 0u;                                       // ready for the next pass / the next call
    local += h[j];
  }
  const uint32_t incl = wave_scan_incl_u32(local);
  if (lane == 63) wave_tot[wv] = incl;
  __syncthreads();
  uint32_t before = incl - local;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) before += (w < wv) ? wave_tot[w] : 0u;
  if (before < k_rem && k_rem <= before + local) {        // exactly one thread
    uint32_t cum = before;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (cum < k_rem && k_rem <= cum + h[j]) {
        const uint32_t digit = (uint32_t)(kRadixBuckets - 1 - (threadIdx.x * 8 + j));
        const uint32_t np = prefix | (digit << radix_shift(pass));
        a.rk_state[2 * r] = np;
        a.rk_state[2 * r + 1] = k_rem - cum;
        if (pass == 2) a.thr[r] = key_value(np);
      }
      cum += h[j];
    }
  }
}

hipError_t launch_topk_radix_select(const KArgs& a, int pass, hipStream_t stream) {
  return launch("topk_radix_select_kernel", topk_radix_select_kernel, dim3((unsigned)(a.rows_t + a.rows_d)), dim3(kThreads),
                stream, a, pass);
}

hipError_t launch_statistics(const KArgs& a, int dtype, bool xf, hipStream_t stream) {
  if (dtype == kDtBF16) return xf ? launch_statistics_bf16_xf(a, stream) : launch_statistics_bf16_plain(a, stream);
  return xf ? launch_statistics_f32_xf(a, stream) : launch_statistics_f32_plain(a, stream);
}

// The drafting stage's draw under truncation: one launch while one workgroup can hold the row
// (65536 logits of bf16, 32768 of fp32: 64 fp32 words per thread).
bool resample_topk_fits(const KArgs& a, int dtype) {
  const int row_one = dtype == kDtBF16 ? 4 * kChunk : 2 * kChunk;
  return a.resample_only && a.top_k > 0 && a.d == nullptr && a.V <= row_one;
}

hipError_t launch_resample_topk(const KArgs& a, int dtype, hipStream_t stream) {
  return dtype == kDtBF16 ? launch_resample_topk_bf16(a, stream) : launch_resample_topk_f32(a, stream);
}

}  // namespace csd
