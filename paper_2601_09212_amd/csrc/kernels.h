// Host <-> kernel interface of the Cool-SD library (internal).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace csd {

// Everything a kernel needs, passed by value.  Pointers are device pointers.
struct KArgs {
  // --- what the statistics kernels read, kept together at the front (two cache lines of the
  //     kernel-argument segment instead of five)
  const void* t;            // target logits (conditional)
  const void* tu;           // target unconditional logits or nullptr
  const void* d;            // draft logits (nullptr: stand-alone resample from p)
  const void* du;           // draft unconditional logits or nullptr
  const int32_t* tokens;    // [B, L]
  float2* part;             // workspace [rows_t + rows_d, c1]  (reference exponent, sum) of every statistics chunk
  float* tok_logit;         // workspace [rows_t + rows_d]      transformed logit of the row's draft token x~_i
  float* thr;               // workspace [rows_t + rows_d]      top-k threshold of every row (top_k > 0)
  int64_t t_sb, t_sl, d_sb, d_sl;          // element strides
  int32_t B, L, V, has_bonus;
  int32_t rows_t, rows_d;   // target rows B*(L+has_bonus), draft rows B*L (0: no draft)
  int32_t c1, top_k;        // statistics chunks per row; top-k (0 = off)
  float cfg_scale, inv_T;
  int32_t win_lo, win_hi;   // statistics pass over the rows of positions [win_lo, win_hi) only (win_hi == 0: all rows)
  // --- the rest
  int64_t om_sb;
  const float* omega;       // [L] or [B, L]
  const float* u_acc;       // [B, L]
  const float* u_res;       // [B]
  int32_t* accept_len;      // [B]
  int32_t* next_token;      // [B]
  float* p_tok;             // [B, L] or nullptr
  float* q_tok;
  float* f;
  float* resid_mass;        // [B] or nullptr
  int32_t resample_mode, resample_only, aligned;
  int32_t stats_only;       // enqueue the statistics pass alone (the benchmark library's timing entry point)
  int32_t early_exit;       // verify: stop reading a sequence's rows at its first rejection (one kernel)
  int32_t exact_draw;       // every draw x ~ G in fp64 (COOL_SD_FLAG_EXACT_DRAW), not only those the fp32 path does not trust
  int32_t stream_loads;     // statistics kernel: input larger than the caches, use nontemporal loads
  int32_t nchunks, nt2;     // sampling kernel: chunks per row, tiles per chunk
  int32_t nt1, chunk1;      // statistics kernel: tiles per chunk, logits per chunk
  float2* rowstat;          // workspace [rows_t + rows_d]      combined statistics (written only when c1 > 4)
  const float2* stat;       // what the sequence kernel reads: part (cs = c1 <= 4) or rowstat (cs = 1)
  int32_t cs;
  int32_t accept_combines;  // long rows: accept_kernel combines the chunk statistics of its own rows (no combine_rows launch)
  float4* seq_stat;         // [B]           statistics of the sampled row (several-chunk path)
  float* chunk_R;           // [B, nchunks]  residual mass per chunk of the sampled row  (nchunks > 1)
  int32_t* ticket;          // [B]           workgroups of the long-row tail launch that have finished their chunks
  int32_t tail_groups;      // workgroups per sequence of that launch
  int32_t windowed;         // verify in rounds of positions that stop reading a sequence after its first rejection
  int32_t* tau_ws;          // [B]           that form's state: -1 while every position so far was accepted, else tau
  // top-k on rows longer than one workgroup: radix-select state in the workspace
  uint32_t* rk_hist;        // [rows_t + rows_d, 2048] digit counts of the current pass
  uint32_t* rk_state;       // [rows_t + rows_d, 2]    key bits fixed so far, rank still to find
  // aggregated acceptance over latent neighbours (nbr == nullptr: off)
  const int32_t* nbr;       // [V, lan_k] neighbour table, nearest first
  int32_t lan_k;
  float lan_lambda;
  float* lan_omega;         // workspace [B, L]: sum over the neighbour set / p(x~_i); read as omega
  int32_t* lan_count;       // workspace [B, L]: members of the set besides x~_i
  float* p_agg_out;         // [B, L] out or nullptr
  int32_t* count_out;       // [B, L] out or nullptr
  int32_t lan_resample;     // 1: resample with Eq. g_lantern
  // diagnostics call only (nchunks = chunks of 8192 logits per row there, has_bonus = 0)
  float* alpha;             // [B, L] out
  float* beta;              // [B, L] out
  float2* diag_part;        // [B*L, nchunks]  (alpha, beta) sums per chunk
};

// Enqueue the kernels of one verify (or stand-alone resample) call.  xf: the logit transform
// (guidance / temperature / top-k) is active.  Returns hipSuccess or the launch error.
hipError_t launch_verify(const KArgs& a, int dtype, bool xf, hipStream_t stream);

// Enqueue the kernels of one diagnostics call (alpha_i, beta_i of every row pair).  local: rows
// are one chunk and need no statistics pass.  have_stats (not with local): the workspace already
// holds the rows' chunk statistics and thresholds, numbered as in a verify call with these
// arguments, so the statistics pass is skipped.
hipError_t launch_diagnostics(const KArgs& a, int dtype, bool xf, bool local, hipStream_t stream, bool have_stats);

// Enqueue the kernels of one cool_sd_verify_diagnostics call on rows of one chunk without top-k
// (every logit read once for both results).
hipError_t launch_verify_diagnostics(const KArgs& a, int dtype, bool xf, hipStream_t stream);

// Checked mode (COOL_SD_FLAG_CHECK_TOKENS), after the kernels of a verify call: sequences that hold a
// draft token outside [0, V) get accept_len = next_token = -1 and resid_mass = 0.
hipError_t launch_check_tokens(const KArgs& a, hipStream_t stream);

// Zero n 32-bit words.
hipError_t launch_zero(uint32_t* p, size_t n, hipStream_t stream);
// benchmark yardstick: streaming read of two buffers (sizes in 16-byte vectors), one word out per workgroup
hipError_t launch_read_probe(const uint4* a, size_t na, const uint4* b, size_t nb, uint32_t* out, hipStream_t stream);
constexpr size_t kProbeVecsPerGroup = 512;   // 8 KiB

// ---------------------------------------------------------------------------------------------
// The pieces the calls above are made of.  Each lives in a translation unit of its own
// (statistics pass, per-sequence step, diagnostics) so that the library builds in parallel; all of
// them only enqueue kernels on `stream`.

// Which launch does the neighbour aggregation of cool_sd_verify_lantern: it rides on the statistics
// launch when it needs no top-k threshold, or when the workgroup that selects a target row's
// threshold can do it (rows of one workgroup); otherwise a launch of its own follows.
inline bool lantern_fused(const KArgs& a) {
  return a.nbr != nullptr && !a.stats_only && (a.top_k == 0 || a.V <= 4 * 16384);
}

// statistics pass (stats_launch.hip): softmax statistics of every row (under top-k: threshold
// selection first), the logit of x~_i per row, and the fused neighbour aggregation
hipError_t launch_statistics(const KArgs& a, int dtype, bool xf, hipStream_t stream);
// cool_sd_resample without a draft under top-k on rows one workgroup holds: one launch
bool resample_topk_fits(const KArgs& a, int dtype);
hipError_t launch_resample_topk(const KArgs& a, int dtype, hipStream_t stream);

// per-sequence step (sequence_launch.hip): everything after the statistics pass
hipError_t launch_sequence(const KArgs& a, int dtype, bool xf, hipStream_t stream);
// whether a long-row call runs its per-sequence step as one launch that finds tau itself (then no
// kernel leaves the combined row statistics in the workspace)
bool tail_in_one_launch(const KArgs& a, int dtype);
hipError_t launch_combine_rows(const KArgs& a, hipStream_t stream);
// the whole verify call per sequence, stopping at the first rejection (COOL_SD_FLAG_EARLY_EXIT)
hipError_t launch_early_exit(const KArgs& a, int dtype, bool xf, hipStream_t stream);
// the same flag on long rows: after the statistics launch of the window [win_lo, win_hi), the accept
// tests of that window for the sequences still without a rejection
hipError_t launch_accept_window(const KArgs& a, int dtype, bool xf, hipStream_t stream);
// cool_sd_resample on rows one workgroup holds, without top-k: one launch
bool resample_whole_fits(const KArgs& a);
hipError_t launch_resample_whole(const KArgs& a, int dtype, bool xf, hipStream_t stream);

// diagnostics (diagnostics_launch.hip)
// one-chunk rows: every logit read once; ver: also leave the verify call's statistics (plus B
// workgroups for the bonus rows)
hipError_t launch_diag_local(const KArgs& a, int dtype, bool xf, bool ver, hipStream_t stream);
// long rows / top-k: chunk sums against the row statistics in the workspace, then their combination
hipError_t launch_diag_chunks(const KArgs& a, int dtype, bool xf, hipStream_t stream);

}  // namespace csd
