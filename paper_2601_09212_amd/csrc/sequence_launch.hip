// Per-sequence step of a verify call (everything after the statistics pass), the early-exit form
// of the whole call, and the one-launch stand-alone resampling on short rows: launch code.
#include "early_exit_kernels.h"
#include "sequence_long.h"
#include "sequence_whole.h"

namespace csd {

// Rows with more than kMaxDirect statistics chunks, where no later kernel combines them itself:
// one wave per row combines the row's chunk statistics into one (reference exponent, sum) pair.
__global__ __launch_bounds__(kThreads) void combine_rows_kernel(const KArgs a) {
  const int r = blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (r >= a.rows_t + a.rows_d) return;
  combine_row_wave(a, r);
}

hipError_t launch_combine_rows(const KArgs& a, hipStream_t stream) {
  const int64_t gridc = (int64_t(a.rows_t) + a.rows_d + kWaves - 1) / kWaves;
  return launch("combine_rows_kernel", combine_rows_kernel, dim3((unsigned)gridc), dim3(kThreads), stream, a);
}

// Eq. f_lantern: the acceptance probability of x~_i uses the probability of its neighbour set
// A(x~_i) = {x~_i} + the longest prefix of its neighbour list (nearest first) whose summed
// probability stays below lambda p_i(x~_i).  Relative to p_i(x~_i) the members weigh
// 2^((l_n - l_x) log2e), which needs no row statistics, so one wave per position gathers the k
// neighbour logits, scans their weights and leaves agg = sum over A / p_i(x~_i) >= 1 where the
// accept test reads its relaxation parameter: Eq. f_lantern is Eq. relax with omega_i = agg.
// Also writes the number of members (for Eq. g_lantern) and the optional outputs.  Launched on
// its own only for rows whose top-k thresholds came from the radix passes.
__global__ __launch_bounds__(kThreads) void lantern_agg_kernel(const KArgs a, int dt, int xf) {
  const int pos = blockIdx.x * kWaves + (threadIdx.x >> 6);       // (b, i)
  if (pos >= a.B * a.L) return;
  const int b = pos / a.L, rt_ = b * (a.L + a.has_bonus) + (pos - b * a.L);
  lantern_agg_position(a, pos, dt, xf != 0, (xf && a.top_k > 0) ? a.thr[rt_] : -INFINITY);
}

// Long rows: the per-sequence step is ONE launch (sequence_tail_kernel) when a row's chunk statistics
// fit one wave and the positions another (rows of up to 524288 logits, draft windows of up to 63
// tokens with the bonus row) and the sampled rows hold at most kTailFusedChunks chunks in all;
// otherwise accept_kernel, sequence_masses_kernel and sequence_select_kernel follow each other.
// The limit is where the two forms cross: the one launch saves two launch gaps and one latency
// chain, but its few dependent loads (tau at the start, the chunk masses and the chosen chunk at
// the end) queue behind its own streaming loads once the launch saturates HBM, which three
// launches, each starting on an idle memory system, do not suffer.
#ifndef CSD_TAIL_MAX
#define CSD_TAIL_MAX 256
#endif
constexpr int64_t kTailFusedChunks = CSD_TAIL_MAX;
bool tail_in_one_launch(const KArgs& a, int dtype) {
  const int kT = dtype == kDtBF16 ? Vec<kDtBF16>::kT : Vec<kDtF32>::kT;
  return !a.resample_only && a.nt2 != kT && a.c1 <= 64 && a.nchunks <= 64 && a.L + a.has_bonus <= kTauRows &&
         int64_t(a.B) * a.nchunks <= kTailFusedChunks;
}

template <int DT, bool XF, bool AL>
static hipError_t launch_sequence_typed(const KArgs& a, hipStream_t stream) {
  constexpr int kT = Vec<DT>::kT;
  hipError_t e;
  const bool one_launch = !a.windowed && tail_in_one_launch(a, DT) && !(AL && !a.lan_resample && a.V <= 2 * kChunk);
  // the long-row kernels of the stand-alone resampling call combine up to 64 chunk statistics themselves
  const bool resample_combines = a.resample_only && a.nt2 != kT && a.c1 <= 64;
  if (a.cs != a.c1 && !a.accept_combines && !one_launch && !resample_combines) {   // rows have many statistics chunks: pre-combine them
    e = launch_combine_rows(a, stream);
    if (e != hipSuccess) return e;
  }
  const dim3 gB((unsigned)a.B), bW(kThreadsW);
  if (a.nbr != nullptr && !lantern_fused(a)) {   // aggregated acceptance on rows whose thresholds came from the radix passes
    const int64_t gl = (int64_t(a.B) * a.L + kWaves - 1) / kWaves;
    e = launch("lantern_agg_kernel", lantern_agg_kernel, dim3((unsigned)gl), dim3(kThreads), stream, a, int(DT), int(XF ? 1 : 0));
    if (e != hipSuccess) return e;
  }
  if (a.nt2 == kT) {          // the sampled row is one chunk: everything per sequence in one workgroup
    if (a.lan_resample) return launch("sequence_whole_kernel", sequence_whole_kernel<DT, XF, AL, true>, gB, bW, stream, a);
    return launch("sequence_whole_kernel", sequence_whole_kernel<DT, XF, AL, false>, gB, bW, stream, a);
  }
  if constexpr (AL) {
    // aligned rows of up to 32768 logits (four statistics chunks, read directly) still fit the
    // registers of one workgroup: the one-launch form
    if (!a.lan_resample && !a.windowed && a.V <= 2 * kChunk)
      return launch("sequence_whole_kernel", sequence_whole_kernel<DT, XF, AL, false, 2>, gB, bW, stream, a);
  }
  if (one_launch) {
    const dim3 gridt((unsigned)(int64_t(a.B) * a.tail_groups));
    if (a.lan_resample) return launch("sequence_tail_kernel", sequence_tail_kernel<DT, XF, AL, kT / 2, true>, gridt, dim3(kThreads), stream, a);
    return launch("sequence_tail_kernel", sequence_tail_kernel<DT, XF, AL, kT / 2, false>, gridt, dim3(kThreads), stream, a);
  }
  if (!a.resample_only && !a.windowed) {     // find tau once per sequence (verification in rounds has done it)
    e = launch("accept_kernel", accept_kernel<DT, XF>, gB, bW, stream, a);
    if (e != hipSuccess) return e;
  }
  const dim3 grid2((unsigned)(int64_t(a.B) * a.nchunks)), b2(kThreads);
  e = a.lan_resample ? launch("sequence_masses_kernel", sequence_masses_kernel<DT, XF, AL, kT / 2, true>, grid2, b2, stream, a)
                     : launch("sequence_masses_kernel", sequence_masses_kernel<DT, XF, AL, kT / 2, false>, grid2, b2, stream, a);
  if (e != hipSuccess) return e;
  if (a.lan_resample) return launch("sequence_select_kernel", sequence_select_kernel<DT, XF, AL, true>, gB, bW, stream, a);
  return launch("sequence_select_kernel", sequence_select_kernel<DT, XF, AL, false>, gB, bW, stream, a);
}

#define CSD_DISPATCH(FN, ...)                                                                              \
  do {                                                                                                     \
    if (dtype == kDtBF16) {                                                                                \
      if (xf) return a.aligned ? FN<kDtBF16, true, true>(__VA_ARGS__) : FN<kDtBF16, true, false>(__VA_ARGS__);   \
      return a.aligned ? FN<kDtBF16, false, true>(__VA_ARGS__) : FN<kDtBF16, false, false>(__VA_ARGS__);   \
    }                                                                                                      \
    if (xf) return a.aligned ? FN<kDtF32, true, true>(__VA_ARGS__) : FN<kDtF32, true, false>(__VA_ARGS__); \
    return a.aligned ? FN<kDtF32, false, true>(__VA_ARGS__) : FN<kDtF32, false, false>(__VA_ARGS__);       \
  } while (0)

hipError_t launch_sequence(const KArgs& a, int dtype, bool xf, hipStream_t stream) {
  CSD_DISPATCH(launch_sequence_typed, a, stream);
}

hipError_t launch_accept_window(const KArgs& a, int dtype, bool xf, hipStream_t stream) {
  const dim3 gB((unsigned)a.B), bk(kThreads);
  const char* what = "accept_window_kernel";
  if (dtype == kDtBF16) return xf ? launch(what, accept_window_kernel<kDtBF16, true>, gB, bk, stream, a)
                                  : launch(what, accept_window_kernel<kDtBF16, false>, gB, bk, stream, a);
  return xf ? launch(what, accept_window_kernel<kDtF32, true>, gB, bk, stream, a)
            : launch(what, accept_window_kernel<kDtF32, false>, gB, bk, stream, a);
}

// Early exit: aligned rows only (the caller checks the conditions of COOL_SD_FLAG_EARLY_EXIT).
hipError_t launch_early_exit(const KArgs& a, int dtype, bool xf, hipStream_t stream) {
  const dim3 gB((unsigned)a.B);
  const char* what = "sequence_early_exit_kernel";
  if (dtype == kDtBF16 && !xf) return launch(what, sequence_early_exit_tile_kernel, gB, dim3(kThreads), stream, a);
  if (dtype == kDtBF16) return launch(what, sequence_early_exit_kernel<kDtBF16, true, 1>, gB, dim3(kThreadsW), stream, a);
  if (xf) return launch(what, sequence_early_exit_kernel<kDtF32, true, 1>, gB, dim3(kThreadsW), stream, a);
  return launch(what, sequence_early_exit_kernel<kDtF32, false, 1>, gB, dim3(kThreadsW), stream, a);
}

// rows that one workgroup holds in registers (16384 logits; 32768 when aligned)
bool resample_whole_fits(const KArgs& a) {
  return a.resample_only && a.top_k == 0 && a.V <= (a.aligned ? 2 * kChunk : kChunk);
}

template <int DT, bool XF, bool AL>
static hipError_t launch_resample_whole_typed(const KArgs& a, hipStream_t stream) {
  const dim3 gB((unsigned)a.B), bW(kThreadsW);
  if (a.V <= kChunk) return launch("resample_whole_kernel", resample_whole_kernel<DT, XF, AL>, gB, bW, stream, a);
  if constexpr (AL) return launch("resample_whole_kernel", resample_whole_kernel<DT, XF, true, 2>, gB, bW, stream, a);
  return hipErrorInvalidValue;    // not reached: resample_whole_fits
}

hipError_t launch_resample_whole(const KArgs& a, int dtype, bool xf, hipStream_t stream) {
  CSD_DISPATCH(launch_resample_whole_typed, a, stream);
}

#undef CSD_DISPATCH

}  // namespace csd
