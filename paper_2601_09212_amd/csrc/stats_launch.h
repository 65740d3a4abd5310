// Launch code of the statistics pass, as templates over (dtype, logit transform, alignment); the
// translation units stats_bf16_xf.hip, stats_bf16_plain.hip, stats_f32_xf.hip and
// stats_f32_plain.hip each instantiate one (dtype, transform) slice so that they compile in parallel.
#pragma once
#include <algorithm>
#include "stats_kernels.h"
#include "topk_kernels.h"

namespace csd {

// one workgroup per row fixes the digit of a radix pass (stats_launch.hip)
hipError_t launch_topk_radix_select(const KArgs& a, int pass, hipStream_t stream);

// Grid of a statistics kernel: (chunks, rows of one sequence, sequences) when the dimensions
// allow it, else one dimension.
inline bool stats_grid3(const KArgs& a, dim3& grid) {
  const int64_t per_t = int64_t(a.L) + a.has_bonus, hi = a.win_hi ? a.win_hi : per_t;
  const int64_t wt = std::min<int64_t>(hi, per_t) - a.win_lo, wd = a.rows_d ? std::min<int64_t>(hi, a.L) - a.win_lo : 0;
  const int64_t per_seq = wt + std::max<int64_t>(wd, 0);
  if (a.B <= 65535 && per_seq <= 65535) {
    grid = dim3((unsigned)a.c1, (unsigned)per_seq, (unsigned)a.B);
    return true;
  }
  grid = dim3((unsigned)((int64_t(a.rows_t) + a.rows_d) * a.c1));
  return false;
}

template <int DT, bool XF, int AL, int NT>
static hipError_t launch_stats(const KArgs& a, hipStream_t stream) {
  dim3 grid;
  const bool g3 = stats_grid3(a, grid);
  if (lantern_fused(a)) {
    const int64_t groups = (int64_t(a.B) * a.L + kWaves - 1) / kWaves;      // one wave per position
    if (g3) {
      const int64_t per_slice = int64_t(grid.x) * grid.y;
      const int64_t slices = (groups + per_slice - 1) / per_slice;
      if (int64_t(grid.z) + slices <= 65535) {
        grid.z += (unsigned)slices;
        return launch("row_stats_kernel", row_stats_kernel<DT, XF, AL, NT, true, true>, grid, dim3(kThreads), stream, a);
      }
      grid = dim3((unsigned)((int64_t(a.rows_t) + a.rows_d) * a.c1));      // too many slices: one dimension
    }
    grid.x += (unsigned)groups;
    return launch("row_stats_kernel", row_stats_kernel<DT, XF, AL, NT, false, true>, grid, dim3(kThreads), stream, a);
  }
  if (g3) return launch("row_stats_kernel", row_stats_kernel<DT, XF, AL, NT, true>, grid, dim3(kThreads), stream, a);
  return launch("row_stats_kernel", row_stats_kernel<DT, XF, AL, NT, false>, grid, dim3(kThreads), stream, a);
}

template <int DT, int kA, int TPB, int ROW>
static hipError_t launch_topk_rows(const KArgs& a, hipStream_t stream) {
  dim3 grid;
  const bool g3 = stats_grid3(a, grid);
  if (g3) grid.x = 1; else grid.x = (unsigned)(a.rows_t + a.rows_d);
  const bool guided = a.tu != nullptr, lanf = lantern_fused(a);
  const char* what = "row_stats_topk_kernel";
#define CSD_TOPK(GD_, G3_)                                                                                          \
  (lanf ? launch(what, row_stats_topk_kernel<DT, kA, TPB, GD_, G3_, ROW, true>, grid, dim3(TPB), stream, a)         \
        : launch(what, row_stats_topk_kernel<DT, kA, TPB, GD_, G3_, ROW, false>, grid, dim3(TPB), stream, a))
  if (g3 && guided) return CSD_TOPK(1, true);
  if (g3) return CSD_TOPK(0, true);
  if (guided) return CSD_TOPK(1, false);
  return CSD_TOPK(0, false);
#undef CSD_TOPK
}

// Statistics pass with the chunk size and load flavour the host chose.
template <int DT, bool XF, bool AL>
static hipError_t launch_stats_any(const KArgs& a, hipStream_t stream) {
  constexpr int kT = Vec<DT>::kT;
  if constexpr (XF) {
    constexpr int kA = AL ? kAligned : kUnaligned;
    if (a.top_k > 0 && a.V > kRowMid) {  // rows beyond one workgroup: three radix passes leave every row's threshold
      dim3 grid;
      const bool g3 = stats_grid3(a, grid);
      const unsigned rows = (unsigned)(a.rows_t + a.rows_d);
      hipError_t e = launch_zero(reinterpret_cast<uint32_t*>(a.rk_hist), size_t(rows) * kRadixBuckets, stream);
      if (e != hipSuccess) return e;
      for (int pass = 0; pass < 3; ++pass) {
        e = g3 ? launch("topk_radix_hist_kernel", topk_radix_hist_kernel<DT, kA, kT / 2, true>, grid, dim3(kThreads), stream, a, pass)
               : launch("topk_radix_hist_kernel", topk_radix_hist_kernel<DT, kA, kT / 2, false>, grid, dim3(kThreads), stream, a, pass);
        if (e != hipSuccess) return e;
        e = launch_topk_radix_select(a, pass, stream);
        if (e != hipSuccess) return e;
      }
    } else if (a.top_k > 0) {            // whole rows, one workgroup each
      if (a.V <= kChunk) return launch_topk_rows<DT, kA, kThreadsK, kChunk>(a, stream);
      // 16384 < V <= 32768: 1024 threads with 32 logits each, statistics per 8192 logits
      if (a.V <= 2 * kChunk) return launch_topk_rows<DT, kA, kThreadsW, 2 * kChunk>(a, stream);
      return launch_topk_rows<DT, kA, kThreadsW, kRowMid>(a, stream);       // up to 65536: 64 logits per thread
    }
  }
  if (AL && a.stream_loads) {   // large read-once input: nontemporal loads
    if (a.nt1 == kT) return launch_stats<DT, XF, kAlignedStream, kT>(a, stream);
    if (a.nt1 == kT / 2) return launch_stats<DT, XF, kAlignedStream, kT / 2>(a, stream);
    return launch_stats<DT, XF, kAlignedStream, kT / 4>(a, stream);
  }
  if (a.nt1 == kT) return launch_stats<DT, XF, AL ? kAligned : kUnaligned, kT>(a, stream);
  if (a.nt1 == kT / 2) return launch_stats<DT, XF, AL ? kAligned : kUnaligned, kT / 2>(a, stream);
  return launch_stats<DT, XF, AL ? kAligned : kUnaligned, kT / 4>(a, stream);
}

template <int DT, int kA>
static hipError_t launch_resample_topk_typed(const KArgs& a, hipStream_t stream) {
  constexpr int kRowOne = DT == kDtBF16 ? 4 * kChunk : 2 * kChunk;
  const dim3 gB((unsigned)a.B);
  const bool guided = a.tu != nullptr;
  const char* what = "resample_topk_kernel";
  if (a.V <= kChunk)
    return guided ? launch(what, resample_topk_kernel<DT, kA, 1>, gB, dim3(kThreadsK), stream, a)
                  : launch(what, resample_topk_kernel<DT, kA, 0>, gB, dim3(kThreadsK), stream, a);
  if (a.V <= 2 * kChunk)
    return guided ? launch(what, resample_topk_kernel<DT, kA, 1, kThreadsW, 2 * kChunk>, gB, dim3(kThreadsW), stream, a)
                  : launch(what, resample_topk_kernel<DT, kA, 0, kThreadsW, 2 * kChunk>, gB, dim3(kThreadsW), stream, a);
  return guided ? launch(what, resample_topk_kernel<DT, kA, 1, kThreadsW, kRowOne>, gB, dim3(kThreadsW), stream, a)
                : launch(what, resample_topk_kernel<DT, kA, 0, kThreadsW, kRowOne>, gB, dim3(kThreadsW), stream, a);
}

// the slices
hipError_t launch_statistics_bf16_xf(const KArgs& a, hipStream_t stream);
hipError_t launch_statistics_bf16_plain(const KArgs& a, hipStream_t stream);
hipError_t launch_statistics_f32_xf(const KArgs& a, hipStream_t stream);
hipError_t launch_statistics_f32_plain(const KArgs& a, hipStream_t stream);
hipError_t launch_resample_topk_bf16(const KArgs& a, hipStream_t stream);
hipError_t launch_resample_topk_f32(const KArgs& a, hipStream_t stream);

}  // namespace csd
