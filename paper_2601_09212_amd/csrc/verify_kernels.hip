// HIP kernels of the Cool-SD verification stage for gfx950 (MI355X).
//
// What is computed (paper notation): for every draft position i of every sequence the
// softmax statistics of the target row p_i and the draft row q_i, the relaxed acceptance
// probability f_i = min{1, omega_i p_i(x~_i)/q_i(x~_i)} (Eq. relax), the accept decision
// u_i <= f_i, the accepted length tau (Algorithm 1) and one draw from the resampling law
// G* = Norm([p - min(q, omega p)]_+) (Eq. opt_G) at the first rejected position, or from
// p_{L+1} when nothing was rejected (Algorithm 1, bonus token).
//
// Two launches per verify call.
//   row_stats_kernel   grid = (chunks, rows of a sequence, sequences).  The HBM-bound pass: every
//                      logit is read once.  A workgroup streams one small chunk (4K-16K logits)
//                      of one row through registers and writes the chunk's softmax statistics
//                      (integer base-2 reference exponent, sum).  No workgroup talks to another;
//                      few registers, so many workgroups per CU keep loads in flight.
//                      Under top-k truncation row_stats_topk_kernel takes its place: one workgroup
//                      holds a whole row (up to 65536 logits) and selects the threshold first.
//   sequence_whole_kernel  grid = B.  Per sequence: combine the chunk statistics of its rows,
//                      accept test at each position, tau = first rejection; then re-read ONLY row
//                      tau+1 (one row pair of 2L+1, usually still in L2 / Infinity Cache), keep it
//                      in registers, form the residual masses and draw x_{tau+1} by a
//                      hierarchical inverse CDF.
// Rows longer than 16384 logits do not fit one workgroup's registers; the second step is then
// split at kernel boundaries: accept_kernel (chunk statistics combined, tau; one workgroup per
// sequence), sequence_masses_kernel (mass of every 8192-logit chunk of the sampled rows,
// streaming) and sequence_select_kernel (pick the chunk that holds u*R, re-read it, inverse
// CDF).  cool_sd_resample on short rows is one launch (resample_whole_kernel, resample_topk_kernel).
// Other entry points add: lantern_agg_position (neighbour aggregation of the LANTERN-style
// acceptance: part of the statistics launch, or lantern_agg_kernel after the radix passes),
// sequence_early_exit_tile_kernel / sequence_early_exit_kernel (the whole call per sequence,
// stopping at the first rejection), diag_kernel (per-position terms of Theorem 2; in
// cool_sd_verify_diagnostics it also plays the statistics pass), and for top-k
// on rows beyond 65536 logits three radix passes (topk_radix_*).
// No workgroup ever waits for another one inside a launch: there are no fences or spin waits
// anywhere, the only global atomics are the integer histogram adds of the radix passes (whose
// sums do not depend on the order), and every output is a pure function of the inputs.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "device_utils.h"
#include "kernels.h"
#include "topk.h"

namespace csd {

enum { kModeOpt = 0, kModeVanilla = 1, kModeP = 2 };
constexpr int kThreadsW = 1024;    // workgroup size of the per-row / per-sequence kernels
constexpr int kWavesW = kThreadsW / 64;


struct Smem {
  float tile_part[kWaves][16];
  float tile_tot[16];
  float scan_tot[kWaves];
  int pick_first[kWaves];
  int pick_last[kWaves];
  int bcast_i;
  float4 rowstat;
};

__device__ __forceinline__ const char* row_ptr(const void* base, int64_t elem_off, int es) {
  return base ? reinterpret_cast<const char*>(base) + elem_off * es : nullptr;
}

// The kernels, by topic (all part of this translation unit; the order matters, later files use
// what earlier ones define):
#include "stats_kernels.h"          // row_stats_kernel, lantern_agg_position
#include "topk_kernels.h"           // row_stats_topk_kernel, resample_topk_kernel, topk_radix_*
#include "sequence_common.h"        // combine_rows_kernel, residual law, eval_position, find_tau
#include "sequence_whole.h"         // sequence_whole_kernel, lantern_agg_kernel
#include "early_exit_kernels.h"     // sequence_early_exit_*kernel, resample_whole_kernel
#include "sequence_long.h"          // accept_kernel, sequence_masses_kernel, sequence_select_kernel
#include "diagnostics_kernels.h"    // diag_kernel, diag_combine_kernel

// ============================================================================ host side: launches

__global__ void zero_words_kernel(uint32_t* p, size_t n) {
  size_t i = size_t(blockIdx.x) * blockDim.x + threadIdx.x;
  const size_t stride = size_t(gridDim.x) * blockDim.x;
  for (; i < n; i += stride) p[i] = 0u;
}

// Launch errors are read with hipGetLastError(), which also reports errors left behind by
// unrelated earlier runtime calls of the host program; those are cleared first.
static hipError_t checked(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) fprintf(stderr, "cool_sd: launch of %s failed: %s\n", what, hipGetErrorString(e));
  return e;
}

// Grid of a statistics kernel: (chunks, rows of one sequence, sequences) when the dimensions
// allow it, else one dimension.
static bool stats_grid3(const KArgs& a, dim3& grid) {
  const int64_t per_seq = int64_t(a.L) + a.has_bonus + (a.rows_d ? a.L : 0);
  if (a.B <= 65535 && per_seq <= 65535) {
    grid = dim3((unsigned)a.c1, (unsigned)per_seq, (unsigned)a.B);
    return true;
  }
  grid = dim3((unsigned)((int64_t(a.rows_t) + a.rows_d) * a.c1));
  return false;
}

// The neighbour aggregation rides on the statistics launch when it needs no top-k threshold.
// Under top-k the workgroup that selects a target row's threshold does it (rows of one workgroup).
static bool lantern_fused(const KArgs& a) {
  return a.nbr != nullptr && !a.stats_only && (a.top_k == 0 || a.V <= 4 * kChunk);
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
        hipLaunchKernelGGL((row_stats_kernel<DT, XF, AL, NT, true, true>), grid, dim3(kThreads), 0, stream, a);
        return checked("row_stats_kernel");
      }
      grid = dim3((unsigned)((int64_t(a.rows_t) + a.rows_d) * a.c1));      // too many slices: one dimension
    }
    grid.x += (unsigned)groups;
    hipLaunchKernelGGL((row_stats_kernel<DT, XF, AL, NT, false, true>), grid, dim3(kThreads), 0, stream, a);
    return checked("row_stats_kernel");
  }
  if (g3)
    hipLaunchKernelGGL((row_stats_kernel<DT, XF, AL, NT, true>), grid, dim3(kThreads), 0, stream, a);
  else
    hipLaunchKernelGGL((row_stats_kernel<DT, XF, AL, NT, false>), grid, dim3(kThreads), 0, stream, a);
  return checked("row_stats_kernel");
}

template <int DT, bool XF, bool AL>
static hipError_t launch_rest(const KArgs& a, hipStream_t stream);

// Statistics pass with the chunk size and load flavour the host chose.
template <int DT, bool XF, bool AL>
static hipError_t launch_stats_any(const KArgs& a, hipStream_t stream) {
  constexpr int kT = Vec<DT>::kT;
  if constexpr (XF) {
    if (a.top_k > 0 && a.V > kRowMid) {  // rows beyond one workgroup: three radix passes leave every row's threshold
      constexpr int kA = AL ? kAligned : kUnaligned;
      dim3 grid;
      const bool g3 = stats_grid3(a, grid);
      const unsigned rows = (unsigned)(a.rows_t + a.rows_d);
      hipError_t e = launch_zero(reinterpret_cast<uint32_t*>(a.rk_hist), size_t(rows) * kRadixBuckets, stream);
      if (e != hipSuccess) return e;
      for (int pass = 0; pass < 3; ++pass) {
        if (g3) hipLaunchKernelGGL((topk_radix_hist_kernel<DT, kA, kT / 2, true>), grid, dim3(kThreads), 0, stream, a, pass);
        else hipLaunchKernelGGL((topk_radix_hist_kernel<DT, kA, kT / 2, false>), grid, dim3(kThreads), 0, stream, a, pass);
        e = checked("topk_radix_hist_kernel");
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(topk_radix_select_kernel, dim3(rows), dim3(kThreads), 0, stream, a, pass);
        e = checked("topk_radix_select_kernel");
        if (e != hipSuccess) return e;
      }
    } else if (a.top_k > 0) {            // whole rows, one workgroup each
      constexpr int kA = AL ? kAligned : kUnaligned;
      dim3 grid;
      const bool g3 = stats_grid3(a, grid);
      if (g3) grid.x = 1; else grid.x = (unsigned)(a.rows_t + a.rows_d);
      const bool guided = a.tu != nullptr;
      const bool lanf = lantern_fused(a);
#define CSD_TOPK_LAUNCH(TPB_, GD_, G3_, ROW_)                                                                             \
  do {                                                                                                                    \
    if (lanf) hipLaunchKernelGGL((row_stats_topk_kernel<DT, kA, TPB_, GD_, G3_, ROW_, true>), grid, dim3(TPB_), 0, stream, a); \
    else hipLaunchKernelGGL((row_stats_topk_kernel<DT, kA, TPB_, GD_, G3_, ROW_, false>), grid, dim3(TPB_), 0, stream, a);      \
  } while (0)
      if (a.V <= kChunk) {
        if (g3 && guided) CSD_TOPK_LAUNCH(kThreadsK, 1, true, kChunk);
        else if (g3) CSD_TOPK_LAUNCH(kThreadsK, 0, true, kChunk);
        else if (guided) CSD_TOPK_LAUNCH(kThreadsK, 1, false, kChunk);
        else CSD_TOPK_LAUNCH(kThreadsK, 0, false, kChunk);
      } else if (a.V <= 2 * kChunk) {    // 16384 < V <= 32768: 1024 threads with 32 logits each, statistics per 8192 logits
        if (g3 && guided) CSD_TOPK_LAUNCH(kThreadsW, 1, true, 2 * kChunk);
        else if (g3) CSD_TOPK_LAUNCH(kThreadsW, 0, true, 2 * kChunk);
        else if (guided) CSD_TOPK_LAUNCH(kThreadsW, 1, false, 2 * kChunk);
        else CSD_TOPK_LAUNCH(kThreadsW, 0, false, 2 * kChunk);
      } else {                           // 32768 < V <= 65536: 64 logits per thread
        if (g3 && guided) CSD_TOPK_LAUNCH(kThreadsW, 1, true, kRowMid);
        else if (g3) CSD_TOPK_LAUNCH(kThreadsW, 0, true, kRowMid);
        else if (guided) CSD_TOPK_LAUNCH(kThreadsW, 1, false, kRowMid);
        else CSD_TOPK_LAUNCH(kThreadsW, 0, false, kRowMid);
      }
#undef CSD_TOPK_LAUNCH
      return checked("row_stats_topk_kernel");
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

template <int DT, bool XF, bool AL>
static hipError_t launch_typed(const KArgs& a, hipStream_t stream, hipEvent_t* ev) {
  (void)hipGetLastError();
  if (ev) (void)hipEventRecord(ev[0], stream);
  if (a.early_exit && !a.stats_only) {   // one launch; there is no separate statistics pass to time
    if (ev) (void)hipEventRecord(ev[1], stream);
    if constexpr (DT == kDtBF16 && !XF)
      hipLaunchKernelGGL(sequence_early_exit_tile_kernel, dim3((unsigned)a.B), dim3(kThreads), 0, stream, a);
    else
      hipLaunchKernelGGL((sequence_early_exit_kernel<DT, XF, 1>), dim3((unsigned)a.B), dim3(kThreadsW), 0, stream, a);
    hipError_t ee = checked("sequence_early_exit_kernel");
    if (ev) (void)hipEventRecord(ev[2], stream);
    return ee;
  }
  if constexpr (XF) {
    // the drafting stage's draw under truncation: one launch while one workgroup can hold the row
    // (65536 logits of bf16, 32768 of fp32: 64 fp32 words per thread)
    constexpr int kRowOne = DT == kDtBF16 ? 4 * kChunk : 2 * kChunk;
    if (a.resample_only && a.top_k > 0 && a.d == nullptr && a.V <= kRowOne && !a.stats_only) {
      constexpr int kA = AL ? kAligned : kUnaligned;
      const dim3 gB((unsigned)a.B);
      const bool guided = a.tu != nullptr;
      if (ev) (void)hipEventRecord(ev[1], stream);
      if (a.V <= kChunk) {
        if (guided) hipLaunchKernelGGL((resample_topk_kernel<DT, kA, 1>), gB, dim3(kThreadsK), 0, stream, a);
        else hipLaunchKernelGGL((resample_topk_kernel<DT, kA, 0>), gB, dim3(kThreadsK), 0, stream, a);
      } else if (a.V <= 2 * kChunk) {
        if (guided) hipLaunchKernelGGL((resample_topk_kernel<DT, kA, 1, kThreadsW, 2 * kChunk>), gB, dim3(kThreadsW), 0, stream, a);
        else hipLaunchKernelGGL((resample_topk_kernel<DT, kA, 0, kThreadsW, 2 * kChunk>), gB, dim3(kThreadsW), 0, stream, a);
      } else {
        if (guided) hipLaunchKernelGGL((resample_topk_kernel<DT, kA, 1, kThreadsW, kRowOne>), gB, dim3(kThreadsW), 0, stream, a);
        else hipLaunchKernelGGL((resample_topk_kernel<DT, kA, 0, kThreadsW, kRowOne>), gB, dim3(kThreadsW), 0, stream, a);
      }
      hipError_t er = checked("resample_topk_kernel");
      if (ev) (void)hipEventRecord(ev[2], stream);
      return er;
    }
  }
  // rows that one workgroup holds in registers (16384 logits; 32768 when aligned): one launch
  const int row_one = AL ? 2 * kChunk : kChunk;
  if (a.resample_only && a.top_k == 0 && a.V <= row_one && !a.stats_only) {
    if (ev) (void)hipEventRecord(ev[1], stream);
    if (a.V <= kChunk) hipLaunchKernelGGL((resample_whole_kernel<DT, XF, AL>), dim3((unsigned)a.B), dim3(kThreadsW), 0, stream, a);
    if constexpr (AL) {
      if (a.V > kChunk) hipLaunchKernelGGL((resample_whole_kernel<DT, XF, true, 2>), dim3((unsigned)a.B), dim3(kThreadsW), 0, stream, a);
    }
    hipError_t er = checked("resample_whole_kernel");
    if (ev) (void)hipEventRecord(ev[2], stream);
    return er;
  }
  hipError_t e = launch_stats_any<DT, XF, AL>(a, stream);
  if (e != hipSuccess || a.stats_only) return e;
  if (ev) (void)hipEventRecord(ev[1], stream);
  e = launch_rest<DT, XF, AL>(a, stream);
  if (ev) (void)hipEventRecord(ev[2], stream);
  return e;
}

// Long rows: the chunk-mass launch finds tau itself when a row's chunk statistics fit one wave and
// the positions another (rows of up to 524288 logits, draft windows of up to 63 tokens), and all
// its workgroups are resident at once -- the search is then latency paid once instead of a
// launch; in a larger grid it would repeat with every round of workgroups (configuration 5,
// 4096 workgroups: 208.5 us with accept_kernel, 212.3 us without).
template <int DT> static bool tau_in_mass_launch(const KArgs& a) {
  return !a.resample_only && a.nt2 != Vec<DT>::kT && a.c1 <= 64 && a.L + a.has_bonus <= kTauRows &&
         int64_t(a.B) * a.nchunks <= 2048;
}

template <int DT, bool XF, bool AL>
static hipError_t launch_rest(const KArgs& a, hipStream_t stream) {
  constexpr int kT = Vec<DT>::kT;
  hipError_t e;
  const bool fuse_tau = tau_in_mass_launch<DT>(a);
  // the long-row kernels of the stand-alone resampling call combine up to 64 chunk statistics themselves
  const bool resample_combines = a.resample_only && a.nt2 != kT && a.c1 <= 64;
  if (a.cs != a.c1 && !a.accept_combines && !fuse_tau && !resample_combines) {   // rows have many statistics chunks: pre-combine them, one wave per row
    const int64_t gridc = (int64_t(a.rows_t) + a.rows_d + kWaves - 1) / kWaves;
    hipLaunchKernelGGL(combine_rows_kernel, dim3((unsigned)gridc), dim3(kThreads), 0, stream, a);
    e = checked("combine_rows_kernel");
    if (e != hipSuccess) return e;
  }
  const unsigned gB = (unsigned)a.B;
  if (a.nbr != nullptr && !lantern_fused(a)) {   // aggregated acceptance on rows whose thresholds came from the radix passes
    const int64_t gl = (int64_t(a.B) * a.L + kWaves - 1) / kWaves;
    hipLaunchKernelGGL(lantern_agg_kernel, dim3((unsigned)gl), dim3(kThreads), 0, stream, a, DT, XF ? 1 : 0);
    e = checked("lantern_agg_kernel");
    if (e != hipSuccess) return e;
  }
  if (a.nt2 == kT) {          // the sampled row is one chunk: everything per sequence in one workgroup
    if (a.lan_resample)
      hipLaunchKernelGGL((sequence_whole_kernel<DT, XF, AL, true>), dim3(gB), dim3(kThreadsW), 0, stream, a);
    else
      hipLaunchKernelGGL((sequence_whole_kernel<DT, XF, AL, false>), dim3(gB), dim3(kThreadsW), 0, stream, a);
    return checked("sequence_whole_kernel");
  }
  if constexpr (AL) {
    // aligned rows of up to 32768 logits (four statistics chunks, read directly) still fit the
    // registers of one workgroup: the one-launch form
    if (!a.lan_resample && a.V <= 2 * kChunk) {
      hipLaunchKernelGGL((sequence_whole_kernel<DT, XF, AL, false, 2>), dim3(gB), dim3(kThreadsW), 0, stream, a);
      return checked("sequence_whole_kernel");
    }
  }
  if (!a.resample_only && !fuse_tau) {     // find tau once per sequence
    hipLaunchKernelGGL((accept_kernel<DT, XF>), dim3(gB), dim3(kThreadsW), 0, stream, a);
    e = checked("accept_kernel");
    if (e != hipSuccess) return e;
  }
  const dim3 grid2((unsigned)(int64_t(a.B) * a.nchunks));
  if (fuse_tau) {
    if (a.lan_resample) hipLaunchKernelGGL((sequence_masses_kernel<DT, XF, AL, kT / 2, true, true>), grid2, dim3(kThreads), 0, stream, a);
    else hipLaunchKernelGGL((sequence_masses_kernel<DT, XF, AL, kT / 2, false, true>), grid2, dim3(kThreads), 0, stream, a);
  } else {
    if (a.lan_resample) hipLaunchKernelGGL((sequence_masses_kernel<DT, XF, AL, kT / 2, true, false>), grid2, dim3(kThreads), 0, stream, a);
    else hipLaunchKernelGGL((sequence_masses_kernel<DT, XF, AL, kT / 2, false, false>), grid2, dim3(kThreads), 0, stream, a);
  }
  e = checked("sequence_masses_kernel");
  if (e != hipSuccess) return e;
  if (a.lan_resample)
    hipLaunchKernelGGL((sequence_select_kernel<DT, XF, AL, true>), dim3(gB), dim3(kThreadsW), 0, stream, a);
  else
    hipLaunchKernelGGL((sequence_select_kernel<DT, XF, AL, false>), dim3(gB), dim3(kThreadsW), 0, stream, a);
  return checked("sequence_select_kernel");
}

template <int DT, bool XF>
static hipError_t launch_al(const KArgs& a, hipStream_t stream, hipEvent_t* ev) {
  return a.aligned ? launch_typed<DT, XF, true>(a, stream, ev) : launch_typed<DT, XF, false>(a, stream, ev);
}

hipError_t launch_verify(const KArgs& a, int dtype, bool xf, hipStream_t stream, hipEvent_t* ev) {
  if (dtype == kDtBF16) return xf ? launch_al<kDtBF16, true>(a, stream, ev) : launch_al<kDtBF16, false>(a, stream, ev);
  return xf ? launch_al<kDtF32, true>(a, stream, ev) : launch_al<kDtF32, false>(a, stream, ev);
}

template <int DT, bool XF, bool AL>
static hipError_t launch_diag_typed(const KArgs& a, bool local, hipStream_t stream, bool have_stats) {
  constexpr int kT = Vec<DT>::kT;
  constexpr int kA = AL ? kAligned : kUnaligned;
  (void)hipGetLastError();
  const int64_t pairs = int64_t(a.B) * a.L;
  if (local) {
    hipLaunchKernelGGL((diag_kernel<DT, XF, kA, kT / 2, true>), dim3((unsigned)pairs), dim3(512), 0, stream, a);
    return checked("diag_kernel (one chunk)");
  }
  hipError_t e = have_stats ? hipSuccess : launch_stats_any<DT, XF, AL>(a, stream);
  if (e != hipSuccess) return e;
  // after a verify call accept_kernel has left the combined rows, unless tau was found by the
  // chunk-mass launch (which combines in LDS only)
  const bool have_rows = have_stats && a.accept_combines && !tau_in_mass_launch<DT>(a);
  if (a.cs != a.c1 && !have_rows) {
    const int64_t gridc = (int64_t(a.rows_t) + a.rows_d + kWaves - 1) / kWaves;
    hipLaunchKernelGGL(combine_rows_kernel, dim3((unsigned)gridc), dim3(kThreads), 0, stream, a);
    e = checked("combine_rows_kernel");
    if (e != hipSuccess) return e;
  }
  // this pass is the last reader of the logits: beyond what the caches hold, nontemporal loads
  const double bytes = double(pairs) * 2.0 * a.V * Vec<DT>::kES * (a.tu ? 2 : 1);
  const dim3 gridd((unsigned)(pairs * a.nchunks));
  if (AL && bytes > 128e6)
    hipLaunchKernelGGL((diag_kernel<DT, XF, AL ? kAlignedStream : kUnaligned, kT / 2, false>), gridd, dim3(kThreads), 0, stream, a);
  else
    hipLaunchKernelGGL((diag_kernel<DT, XF, kA, kT / 2, false>), gridd, dim3(kThreads), 0, stream, a);
  e = checked("diag_kernel");
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(diag_combine_kernel, dim3((unsigned)((pairs + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                     stream, a);
  return checked("diag_combine_kernel");
}

// cool_sd_verify_diagnostics on rows of one chunk without top-k: the pair kernel (statistics,
// token logits, alpha, beta; B more workgroups for the bonus rows), then the per-sequence kernel.
template <int DT, bool XF, bool AL>
static hipError_t launch_verify_diag_typed(const KArgs& a, hipStream_t stream) {
  constexpr int kT = Vec<DT>::kT;
  constexpr int kA = AL ? kAligned : kUnaligned;
  (void)hipGetLastError();
  const int64_t groups = int64_t(a.B) * a.L + (a.has_bonus ? a.B : 0);
  hipLaunchKernelGGL((diag_kernel<DT, XF, kA, kT / 2, true, true>), dim3((unsigned)groups), dim3(512), 0, stream, a);
  hipError_t e = checked("diag_kernel (with the verify call's statistics)");
  if (e != hipSuccess) return e;
  return launch_rest<DT, XF, AL>(a, stream);
}

hipError_t launch_verify_diagnostics(const KArgs& a, int dtype, bool xf, hipStream_t stream) {
  if (dtype == kDtBF16) {
    if (xf) return a.aligned ? launch_verify_diag_typed<kDtBF16, true, true>(a, stream)
                             : launch_verify_diag_typed<kDtBF16, true, false>(a, stream);
    return a.aligned ? launch_verify_diag_typed<kDtBF16, false, true>(a, stream)
                     : launch_verify_diag_typed<kDtBF16, false, false>(a, stream);
  }
  if (xf) return a.aligned ? launch_verify_diag_typed<kDtF32, true, true>(a, stream)
                           : launch_verify_diag_typed<kDtF32, true, false>(a, stream);
  return a.aligned ? launch_verify_diag_typed<kDtF32, false, true>(a, stream)
                   : launch_verify_diag_typed<kDtF32, false, false>(a, stream);
}

hipError_t launch_diagnostics(const KArgs& a, int dtype, bool xf, bool local, hipStream_t stream, bool have_stats) {
  if (dtype == kDtBF16) {
    if (xf) return a.aligned ? launch_diag_typed<kDtBF16, true, true>(a, local, stream, have_stats)
                             : launch_diag_typed<kDtBF16, true, false>(a, local, stream, have_stats);
    return a.aligned ? launch_diag_typed<kDtBF16, false, true>(a, local, stream, have_stats)
                     : launch_diag_typed<kDtBF16, false, false>(a, local, stream, have_stats);
  }
  if (xf) return a.aligned ? launch_diag_typed<kDtF32, true, true>(a, local, stream, have_stats)
                           : launch_diag_typed<kDtF32, true, false>(a, local, stream, have_stats);
  return a.aligned ? launch_diag_typed<kDtF32, false, true>(a, local, stream, have_stats)
                   : launch_diag_typed<kDtF32, false, false>(a, local, stream, have_stats);
}

// Streaming-read yardstick (cool_sd_profile_read_probe): workgroup g reads 512 consecutive
// vectors of buffer a (g < ga) or b, two loads per thread in flight, and leaves the
// exclusive-or of what it read.
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
  (void)hipGetLastError();
  hipLaunchKernelGGL(read_probe_kernel, dim3((unsigned)(ga + gb)), dim3(kThreads), 0, stream, a, na, b, nb, (unsigned)ga, out);
  return checked("read_probe_kernel");
}

hipError_t launch_zero(uint32_t* p, size_t n, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  (void)hipGetLastError();
  hipLaunchKernelGGL(zero_words_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, p, n);
  return checked("zero_words_kernel");
}

}  // namespace csd
