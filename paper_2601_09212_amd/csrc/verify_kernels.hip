// Cool-SD verification stage for gfx950 (MI355X): which kernels a call enqueues, and the few
// kernels that belong to no other translation unit.
//
// What is computed (paper notation): for every draft position i of every sequence the
// softmax statistics of the target row p_i and the draft row q_i, the relaxed acceptance
// probability f_i = min{1, omega_i p_i(x~_i)/q_i(x~_i)} (Eq. relax), the accept decision
// u_i <= f_i, the accepted length tau (Algorithm 1) and one draw from the resampling law
// G* = Norm([p - min(q, omega p)]_+) (Eq. opt_G) at the first rejected position, or from
// p_{L+1} when nothing was rejected (Algorithm 1, bonus token).
//
// A verify call is a statistics pass followed by a per-sequence step.
//   statistics pass (stats_launch.hip, stats_kernels.h, topk_kernels.h)
//       row_stats_kernel: grid = (chunks, rows of a sequence, sequences).  The HBM-bound pass: every
//       logit is read once.  A workgroup streams one small chunk (4K-16K logits) of one row through
//       registers and writes the chunk's softmax statistics (integer base-2 reference exponent,
//       sum).  No workgroup talks to another; few registers, so many workgroups per compute unit
//       keep loads in flight.  Under top-k truncation row_stats_topk_kernel takes its place: one
//       workgroup holds a whole row (up to 65536 logits) and selects the threshold first; longer
//       rows take three radix passes (topk_radix_*) before the ordinary kernel.
//   per-sequence step (sequence_launch.hip, sequence_whole.h, sequence_long.h)
//       rows of one chunk: sequence_whole_kernel, grid = B.  Combine the chunk statistics of the
//       sequence's rows, accept test at each position, tau = first rejection; then re-read ONLY
//       row tau+1 (one row pair of 2L+1, usually still in L2 / Infinity Cache), keep it in
//       registers, form the residual masses and draw x_{tau+1} by a hierarchical inverse CDF.
//       longer rows: accept_kernel (tau; one workgroup per sequence), sequence_masses_kernel (mass
//       of every 8192-logit chunk of the sampled rows, streaming) and sequence_select_kernel (the
//       chunk that holds u*R, re-read, inverse CDF); on small batches the three are one launch,
//       sequence_tail_kernel, whose last workgroup per sequence (a ticket) does the selection.
//   A draw that fp32 cannot resolve is re-done in fp64 inside the same kernel (exact_draw.h).
// Other forms: COOL_SD_FLAG_EARLY_EXIT (sequence_early_exit_*_kernel: the whole call per
// sequence on rows of one chunk; longer rows: rounds of positions, launch_verify below);
// cool_sd_resample on short rows is one launch (resample_whole_kernel, resample_topk_kernel);
// lantern_agg_position (neighbour aggregation of the LANTERN-style acceptance: part of the
// statistics launch, or lantern_agg_kernel after the radix passes); diag_kernel (per-position
// terms of Theorem 2; in cool_sd_verify_diagnostics it also plays the statistics pass).
// No workgroup ever spins or waits for another one.  Global atomics: the integer histogram adds
// of the radix passes (order-independent sums) and the relaxed ticket of sequence_tail_kernel;
// there are no fences.  Every output is a pure function of the inputs.
#include <algorithm>
#include "kernel_common.h"

namespace csd {

__global__ void zero_words_kernel(uint32_t* p, size_t n) {
  size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  const size_t stride = size_t(gridDim.x) * blockDim.x;
  for (; i < n; i += stride) p[i] = 0u;
}

// Checked mode: the kernels clamp every draft token they use as an address, so a token outside
// [0, V) never makes them read outside a row, but the sequence's results mean nothing.  This
// marks such sequences: one thread per sequence walks its L tokens.
__global__ __launch_bounds__(kThreads) void check_tokens_kernel(const KArgs a) {
  const int b = blockIdx.x * kThreads + threadIdx.x;
  if (b >= a.B) return;
  bool bad = false;
  for (int i = 0; i < a.L; ++i) {
    const int x = a.tokens[int64_t(b) * a.L + i];
    bad = bad || x < 0 || x >= a.V;
  }
  if (bad) {
    a.accept_len[b] = -1;
    a.next_token[b] = -1;
    if (a.resid_mass) a.resid_mass[b] = 0.f;
  }
}

hipError_t launch_check_tokens(const KArgs& a, hipStream_t stream) {
  return launch("check_tokens_kernel", check_tokens_kernel, dim3((unsigned)((a.B + kThreads - 1) / kThreads)), dim3(kThreads),
                stream, a);
}

hipError_t launch_verify(const KArgs& a, int dtype, bool xf, hipStream_t stream) {
  if (a.early_exit && !a.stats_only) return launch_early_exit(a, dtype, xf, stream);   // one launch
  if (!a.stats_only) {
    // stand-alone resampling on rows that one workgroup holds: one launch
    if (xf && resample_topk_fits(a, dtype)) return launch_resample_topk(a, dtype, stream);
    if (resample_whole_fits(a)) return launch_resample_whole(a, dtype, xf, stream);
  }
  if (a.windowed && !a.stats_only) {
    // rounds of 1, 1, 2, 4, ... positions, at most 63; the bonus row rides with the last round
    KArgs w = a;
    for (int lo = 0, n = 1; lo < a.L;) {
      const int hi = std::min(lo + n, (int)a.L);
      w.win_lo = lo;
      w.win_hi = hi == a.L ? a.L + a.has_bonus : hi;
      hipError_t e = launch_statistics(w, dtype, xf, stream);
      if (e == hipSuccess) e = launch_accept_window(w, dtype, xf, stream);
      if (e != hipSuccess) return e;
      n = hi == 1 ? 1 : std::min(2 * n, 63);
      lo = hi;
    }
    return launch_sequence(a, dtype, xf, stream);
  }
  hipError_t e = launch_statistics(a, dtype, xf, stream);
  if (e != hipSuccess || a.stats_only) return e;
  return launch_sequence(a, dtype, xf, stream);
}

hipError_t launch_diagnostics(const KArgs& a, int dtype, bool xf, bool local, hipStream_t stream, bool have_stats) {
  if (local) return launch_diag_local(a, dtype, xf, /*ver=*/false, stream);
  hipError_t e = have_stats ? hipSuccess : launch_statistics(a, dtype, xf, stream);
  if (e != hipSuccess) return e;
  // after a verify call accept_kernel has left the combined rows, unless the per-sequence step ran
  // as one launch (which combines in LDS only)
  const bool have_rows = have_stats && a.accept_combines && !tail_in_one_launch(a, dtype);
  if (a.cs != a.c1 && !have_rows) {
    e = launch_combine_rows(a, stream);
    if (e != hipSuccess) return e;
  }
  return launch_diag_chunks(a, dtype, xf, stream);
}

// cool_sd_verify_diagnostics on rows of one chunk without top-k: the pair kernel (statistics,
// token logits, alpha, beta; B more workgroups for the bonus rows), then the per-sequence kernel.
hipError_t launch_verify_diagnostics(const KArgs& a, int dtype, bool xf, hipStream_t stream) {
  hipError_t e = launch_diag_local(a, dtype, xf, /*ver=*/true, stream);
  if (e != hipSuccess) return e;
  return launch_sequence(a, dtype, xf, stream);
}

// Streaming-read yardstick of the benchmark library: workgroup g reads 512 consecutive vectors of
// buffer a (g < ga) or b, two loads per thread in flight, and leaves the exclusive-or of what it
// read.
__global__ __launch_bounds__(kThreads) void read_probe_kernel(const uint4* __restrict__ a, size_t na,
                                                             const uint4* __restrict__ b, size_t nb, unsigned ga,
                                                             uint32_t* __restrict__ out) {
  __shared__ uint32_t red[kWaves];
  const bool first = blockIdx.x < ga;
  const uint4* src = first ? a : b;
  const size_t n = first ? na : nb;
  const size_t base = size_t(first ? blockIdx.x : blockIdx.x - ga) * kProbeVecsPerGroup;
  size_t i0 = base + threadIdx.x, i1 = base + kThreads + threadIdx.x;
  const uint4 v0 = src[i0 < n ? i0 : n - 1], v1 = src[i1 < n ? i1 : n - 1];
  uint32_t x = v0.x ^ v0.y ^ v0.z ^ v0.w ^ v1.x ^ v1.y ^ v1.z ^ v1.w;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x ^= __shfl_xor(x, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = x;
  __syncthreads();
  if (threadIdx.x == 0) out[blockIdx.x] = red[0] ^ red[1] ^ red[2] ^ red[3];
}

hipError_t launch_read_probe(const uint4* a, size_t na, const uint4* b, size_t nb, uint32_t* out, hipStream_t stream) {
  const size_t ga = (na + kProbeVecsPerGroup - 1) / kProbeVecsPerGroup, gb = (nb + kProbeVecsPerGroup - 1) / kProbeVecsPerGroup;
  return launch("read_probe_kernel", read_probe_kernel, dim3((unsigned)(ga + gb)), dim3(kThreads), stream, a, na, b, nb,
                (unsigned)ga, out);
}

hipError_t launch_zero(uint32_t* p, size_t n, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  return launch("zero_words_kernel", zero_words_kernel, dim3((unsigned)blocks), dim3(256), stream, p, n);
}

}  // namespace csd
