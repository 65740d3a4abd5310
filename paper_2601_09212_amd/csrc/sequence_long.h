// Per-sequence step of a verify call on rows longer than 32768 logits (tau, chunk masses, selection).
#pragma once
#include "sequence_whole.h"

namespace csd {

// ============================================================================ kernel 2, long rows
// Rows too long for one workgroup's registers: tau, then the draw x_{tau+1} from the resampling law
// of the sampled row (Eq. opt_G / Eq. g_tsd / p_{L+1}), cut at kernel boundaries.
//   accept_kernel           grid = B, 1024 threads.  tau of every sequence.
//   sequence_masses_kernel  grid = B x C, 256 threads.  Rows of C chunks of 8192 logits:
//                           workgroup (b, c) writes the mass of chunk c (the bandwidth part: the
//                           row pair is streamed once).
//   sequence_select_kernel  grid = B, 1024 threads.  Walks the C chunk masses, loads the chunk that
//                           holds u*R and finds the token in it.
//   sequence_tail_kernel    grid = B x G, 256 threads.  The three above in one launch, for calls
//                           whose sampled rows hold few chunks in all (small batches).
//   accept_window_kernel    grid = B, 256 threads.  COOL_SD_FLAG_EARLY_EXIT: tau by rounds of positions.

// What both kernels need to know about the row that sequence b samples from.
struct SampledRow {
  int j;                  // position tau+1 (0-based row index), L for the bonus row
  bool bonus, none;       // none: tau == L without a bonus row, nothing to sample
  int rt_, rd_;           // row numbers in the statistics arrays
  const char *t_c, *t_u, *d_c, *d_u;
  float thr_t, thr_d, omega;
};

// omega_known: the caller already holds omega of the sampled position (NaN: load it here).
template <int DT, bool XF>
__device__ __forceinline__ SampledRow sampled_row(const KArgs& a, int b, int tau, float omega_known = NAN) {
  constexpr int kES = Vec<DT>::kES;
  SampledRow r;
  const int rps = a.L + a.has_bonus;
  const bool masked = XF && a.top_k > 0;
  r.j = a.resample_only ? 0 : tau;
  r.none = !a.resample_only && r.j >= a.L && !a.has_bonus;
  r.bonus = a.resample_only ? (a.d == nullptr) : (r.j == a.L);
  r.rt_ = b * rps + r.j;
  r.rd_ = a.rows_t + b * a.L + r.j;
  r.t_c = row_ptr(a.t, int64_t(b) * a.t_sb + int64_t(r.j) * a.t_sl, kES);
  r.t_u = row_ptr(a.tu, int64_t(b) * a.t_sb + int64_t(r.j) * a.t_sl, kES);
  r.d_c = r.bonus ? nullptr : row_ptr(a.d, int64_t(b) * a.d_sb + int64_t(r.j) * a.d_sl, kES);
  r.d_u = r.bonus ? nullptr : row_ptr(a.du, int64_t(b) * a.d_sb + int64_t(r.j) * a.d_sl, kES);
  r.thr_t = r.thr_d = -INFINITY;
  r.omega = 1.f;
  if (!r.none) {
    if (masked) r.thr_t = a.thr[r.rt_];
    if (masked && !r.bonus) r.thr_d = a.thr[r.rd_];
    if (!r.bonus) r.omega = omega_known == omega_known ? omega_known : a.omega[int64_t(b) * a.om_sb + r.j];
  }
  return r;
}

// Statistics (Ct, St, Cd, Sd) of the sampled row: left by accept_kernel, or, for the stand-alone
// resampling call, combined here -- by the first wave straight from the chunk statistics (lane c
// takes chunk c) when a row has at most 64 of them, else by one thread from the combined row
// statistics that combine_rows_kernel left.  All threads must call it.
__device__ __forceinline__ float4 sampled_row_stats(const KArgs& a, int b, const SampledRow& r, float4* slot) {
  if (!a.resample_only) return a.seq_stat[b];
  if (a.c1 <= 64) {
    if (threadIdx.x < 64) {
      const int lane = threadIdx.x, cl = lane < a.c1 ? lane : 0;
      const float2 vt = a.part[int64_t(r.rt_) * a.c1 + cl];
      const float2 vd = a.part[int64_t(r.bonus ? r.rt_ : r.rd_) * a.c1 + cl];     // a bonus row has no draft: read and dropped
      const bool in = lane < a.c1;
      const float ct = in ? vt.x : kRefFloor, cd = (in && !r.bonus) ? vd.x : kRefFloor;
      const float Ct = wave_max(ct), Cd = wave_max(cd);
      const float St = wave_sum((in ? vt.y : 0.f) * exp2_fast(ct - Ct));
      const float Sd = wave_sum(((in && !r.bonus) ? vd.y : 0.f) * exp2_fast(cd - Cd));
      if (lane == 0) *slot = make_float4(Ct, St, Cd, Sd);
    }
  } else if (threadIdx.x == 0) {
    float Ct, St, Cd = kRefFloor, Sd = 0.f;
    combine_row(a, r.rt_, Ct, St);
    if (!r.bonus) combine_row(a, r.rd_, Cd, Sd);
    *slot = make_float4(Ct, St, Cd, Sd);
  }
  __syncthreads();
  return *slot;
}

// Eq. g_lantern for a thread that owns tokens first_tok .. first_tok + span - 1 (span <= 32) of
// the row of position j: which of them belong to the rejected token's neighbour set, and where the
// rejected token itself sits (-1: not here).
__device__ __forceinline__ LanPatch lan_patch_span(const KArgs& a, int b, int j, float omega, int64_t first_tok, int span) {
  LanPatch lp{0u, -1, 1.f};
  const int xd = min(max(a.tokens[int64_t(b) * a.L + j], 0), a.V - 1);
  const int m = a.lan_count[int64_t(b) * a.L + j];
  lp.agg = omega;                                     // sum over the set / p(x~_j), from lantern_agg_position
  const int64_t dx = int64_t(xd) - first_tok;
  if (dx >= 0 && dx < span) lp.aggpos = (int)dx;
  const int32_t* row = a.nbr + int64_t(xd) * a.lan_k;
  int taken = 0;
  for (int jj = 0; jj < a.lan_k && taken < m; ++jj) {   // the first m valid neighbours are the members
    const int n = row[jj];
    if (n < 0 || n >= a.V || n == xd) continue;
    ++taken;
    const int64_t dn = int64_t(n) - first_tok;
    if (dn >= 0 && dn < span) lp.zmask |= 1u << (int)dn;
  }
  return lp;
}

// Eq. g_lantern for a thread of a 256-thread workgroup that holds a chunk of `span` tokens from
// `base` on in the tile layout (element e of tile t of thread tid is token
// base + (t*256 + tid)*kE + e, patch bit t*kE + e): which of its tokens belong to the rejected
// token's neighbour set, and where the rejected token itself sits (-1: not here).
template <int kE>
__device__ __forceinline__ LanPatch lan_patch_tile(const KArgs& a, int b, int j, float omega, int64_t base, int span) {
  LanPatch lp{0u, -1, 1.f};
  auto slot = [&](int tokn) -> int {              // bit of token tokn in this thread, or -1
    const int64_t rel = int64_t(tokn) - base;
    if (rel < 0 || rel >= span) return -1;
    const int vec = int(rel) / kE;
    if ((vec & (kThreads - 1)) != (int)threadIdx.x) return -1;
    return (vec / kThreads) * kE + (int(rel) - vec * kE);
  };
  const int xd = min(max(a.tokens[int64_t(b) * a.L + j], 0), a.V - 1);
  const int m = a.lan_count[int64_t(b) * a.L + j];
  lp.agg = omega;                                     // sum over the set / p(x~_j), from lantern_agg_position
  lp.aggpos = slot(xd);
  const int32_t* row = a.nbr + int64_t(xd) * a.lan_k;
  int taken = 0;
  for (int jj = 0; jj < a.lan_k && taken < m; ++jj) {   // the first m valid neighbours are the members
    const int n = row[jj];
    if (n < 0 || n >= a.V || n == xd) continue;
    ++taken;
    const int sl = slot(n);
    if (sl >= 0) lp.zmask |= 1u << sl;
  }
  return lp;
}

// tau of sequence b found by a 256-thread workgroup from the chunk statistics of the sequence's
// rows (at most 64 chunks per row, at most kTauRows positions, the bonus row included), so that
// sequence_tail_kernel needs no accept_kernel before it: every workgroup of a sequence finds the
// same tau for itself (same code, same inputs), the one with emit = true writes accept_len and
// the per-position outputs.
//   wave w combines rows w, w+4, ... -- lane c takes chunk c, eight rows' loads in flight, then a
//   wave maximum and a wave sum per row -- into LDS; one barrier; lane i of wave 0 runs the accept
//   test of position i (its other inputs were requested at the very start); ballot; one barrier.
constexpr int kTauRows = 64;
struct SmemTau {
  float2 st[2 * kTauRows];       // (reference exponent, sum): target rows 0 .. L(+1)-1, then the draft rows
  float4 rowstat;
  float omega;                   // omega of the sampled position (1 for the bonus row)
  int tau;
};
__device__ __forceinline__ int find_tau_from_parts(const KArgs& a, int b, bool emit, SmemTau& sm) {
  constexpr int kBatch = 8;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int rps = a.L + a.has_bonus, nrows = rps + a.L;
  const bool mine = wv == 0 && lane < rps;              // this lane evaluates position `lane`
  const bool has_draft = lane < a.L;
  const int id = has_draft ? lane : a.L - 1;
  float lt = 0.f, ld = 0.f, omega = 0.f, u = 0.f;
  if (mine) {
    lt = a.tok_logit[b * rps + lane];
    ld = a.tok_logit[a.rows_t + b * a.L + id];
    omega = a.omega[int64_t(b) * a.om_sb + id];
    u = a.u_acc[int64_t(b) * a.L + id];
  }
  const int cl = lane < a.c1 ? lane : 0;
  for (int q0 = wv; q0 < nrows; q0 += kWaves * kBatch) {
    float2 v[kBatch];
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      const int q = min(q0 + k * kWaves, nrows - 1);      // clamped: a row past the end is read and dropped
      const int row = q < rps ? b * rps + q : a.rows_t + b * a.L + (q - rps);
      v[k] = a.part[int64_t(row) * a.c1 + cl];
    }
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      const int q = q0 + k * kWaves;
      const float cx = lane < a.c1 ? v[k].x : kRefFloor, sx = lane < a.c1 ? v[k].y : 0.f;
      const float m = wave_max(cx);
      const float t = wave_sum(sx * exp2_fast(cx - m));
      if (lane == 0 && q < nrows) sm.st[q] = make_float2(m, t);
    }
  }
  __syncthreads();
  if (wv == 0) {
    bool rej = false;
    float Ct = kRefFloor, St = 0.f, Cd = kRefFloor, Sd = 0.f;
    if (mine) {
      const float2 t2 = sm.st[lane], d2 = sm.st[rps + id];
      Ct = t2.x; St = t2.y; Cd = d2.x; Sd = d2.y;
      rej = accept_test(a, b, lane, emit, has_draft, Ct, St, Cd, Sd, lt, ld, omega, u);
      if (!has_draft) { Cd = kRefFloor; Sd = 0.f; }       // the bonus row stands alone
    }
    const unsigned long long br = __ballot(rej);
    const int w = br ? __ffsll((long long)br) - 1 : a.L;
    if (lane == w) {                                          // position w, or the bonus row when w == L
      sm.rowstat = make_float4(Ct, St, Cd, Sd);
      sm.omega = has_draft ? omega : 1.f;
    }
    if (lane == 0) {
      sm.tau = w;
      if (emit) a.accept_len[b] = w;
    }
  }
  __syncthreads();
  return sm.tau;
}

// Rows of many statistics chunks, on the path that reads combined row statistics back from the
// workspace: combine the chunks of sequence b's rows, one wave per row (what combine_rows_kernel
// does for all rows).  All 1024 threads of the workgroup must call it.
__device__ __forceinline__ void combine_sequence_rows(const KArgs& a, int b) {
  const int rps = a.L + a.has_bonus, nrows = rps + a.L;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  auto row_of = [&](int q) { return q < rps ? b * rps + q : a.rows_t + b * a.L + (q - rps); };
  if (a.c1 <= 64) {
    // lane c takes chunk c; the loads of up to four of this wave's rows are in flight together,
    // so a wave with several rows pays one memory round trip, not one per row
    constexpr int kBatch = 4;
    const int cl = lane < a.c1 ? lane : 0;
    for (int q0 = wv; q0 < nrows; q0 += kWavesW * kBatch) {
      float2 v[kBatch];
#pragma unroll
      for (int k = 0; k < kBatch; ++k) v[k] = a.part[int64_t(row_of(min(q0 + k * kWavesW, nrows - 1))) * a.c1 + cl];
#pragma unroll
      for (int k = 0; k < kBatch; ++k) {
        const int q = q0 + k * kWavesW;
        const float cx = lane < a.c1 ? v[k].x : kRefFloor, sx = lane < a.c1 ? v[k].y : 0.f;
        const float m = wave_max(cx);
        const float t = wave_sum(sx * exp2_fast(cx - m));
        if (lane == 0 && q < nrows) a.rowstat[row_of(q)] = make_float2(m, t);
      }
    }
  } else {
    for (int q = wv; q < nrows; q += kWavesW) combine_row_wave(a, row_of(q));
  }
  __syncthreads();          // the rows' statistics are visible to the whole workgroup
}

// Middle kernel of the several-chunk path when the chunk-mass grid is large: one workgroup per
// sequence finds tau and leaves accept_len[b] and the sampled row's statistics for the kernels
// that follow.
template <int DT, bool XF>
__global__ __launch_bounds__(kThreadsW) void accept_kernel(const KArgs a) {
  // (find_tau_from_parts with sixteen waves was measured here too: 5.3 us against 4.8 us on
  // configuration 5 -- with one or two rows per wave its batches of eight are mostly padding)
  __shared__ SmemW sm;
  const int b = blockIdx.x;
  if (a.accept_combines) combine_sequence_rows(a, b);
  find_tau<DT, XF, kThreadsW>(a, b, true, sm.pick, &sm.rowstat);
  if (threadIdx.x == 0) a.seq_stat[b] = sm.rowstat;
}

// COOL_SD_FLAG_EARLY_EXIT on long rows: Algorithm 1's `break`, taken between launches.  The call
// walks the draft window in rounds of 1, 1, 2, 4, ... positions (at most 63, the bonus row rides with
// the last round); a round is a statistics launch over the rows of its positions -- workgroups of a
// sequence that already has its rejection return at once -- followed by this kernel, which runs the
// accept tests of the round for the sequences still without a rejection: 256 threads per sequence,
// wave w combines the chunk statistics of rows w, w+4, ... of the round (lane c takes chunk c: rows
// of at most 64 chunks), then lane i of the first wave tests position win_lo + i.  A sequence whose
// tau is now known gets accept_len and the statistics of the row it samples from, as accept_kernel
// would leave them; the per-position outputs of positions after the rejected one are NaN (never
// evaluated).  tau_ws[b] stays -1 while the sequence has no rejection.
template <int DT, bool XF>
__global__ __launch_bounds__(kThreads) void accept_window_kernel(const KArgs a) {
  __shared__ SmemTau sm;
  const int b = blockIdx.x, lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int rps = a.L + a.has_bonus;
  const int lo = a.win_lo, ht = min(a.win_hi, rps), hd = min(a.win_hi, a.L);
  const int nt = ht - lo, nd = max(hd - lo, 0), nrows = nt + nd;
  const bool last = a.win_hi >= rps;
  if (lo > 0 && a.tau_ws[b] >= 0) {           // rejected in an earlier round
    for (int i = lo + threadIdx.x; i < hd; i += kThreads) {
      const int64_t o = int64_t(b) * a.L + i;
      if (a.p_tok) a.p_tok[o] = NAN;
      if (a.q_tok) a.q_tok[o] = NAN;
      if (a.f) a.f[o] = NAN;
    }
    return;
  }
  const int pos = lo + lane;
  const bool mine = wv == 0 && lane < nt;               // this lane tests position `pos`
  const bool has_draft = pos < a.L;
  float lt = 0.f, ld = 0.f, omega = 1.f, u = 0.f;
  if (mine) {
    lt = a.tok_logit[b * rps + pos];
    if (has_draft) {
      ld = a.tok_logit[a.rows_t + b * a.L + pos];
      omega = a.omega[int64_t(b) * a.om_sb + pos];
      u = a.u_acc[int64_t(b) * a.L + pos];
    }
  }
  const int cl = lane < a.c1 ? lane : 0;
  constexpr int kBatch = 4;                             // rows whose loads a wave has in flight together
  for (int q0 = wv; q0 < nrows; q0 += kWaves * kBatch) {
    float2 v[kBatch];
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      const int q = min(q0 + k * kWaves, nrows - 1);      // clamped: a row past the end is read and dropped
      const int row = q < nt ? b * rps + lo + q : a.rows_t + b * a.L + lo + (q - nt);
      v[k] = a.part[int64_t(row) * a.c1 + cl];
    }
#pragma unroll
    for (int k = 0; k < kBatch; ++k) {
      const int q = q0 + k * kWaves;
      const float cx = lane < a.c1 ? v[k].x : kRefFloor, sx = lane < a.c1 ? v[k].y : 0.f;
      const float m = wave_max(cx);
      const float t = wave_sum(sx * exp2_fast(cx - m));
      if (lane == 0 && q < nrows) sm.st[q] = make_float2(m, t);
    }
  }
  __syncthreads();
  if (wv != 0) return;
  bool rej = false;
  float Ct = kRefFloor, St = 0.f, Cd = kRefFloor, Sd = 0.f;
  if (mine) {
    const float2 t2 = sm.st[lane];
    Ct = t2.x; St = t2.y;
    if (has_draft) {
      const float2 d2 = sm.st[nt + lane];
      Cd = d2.x; Sd = d2.y;
    }
    rej = accept_test(a, b, pos, true, has_draft, Ct, St, Cd, Sd, lt, ld, omega, u);
  }
  const unsigned long long br = __ballot(rej);
  const int w = br ? __ffsll((long long)br) - 1 : (last ? a.L - lo : -1);    // lane of the sampled row, -1: none yet
  if (w >= 0 && mine && has_draft && lane > w) {        // positions after the rejected one
    const int64_t o = int64_t(b) * a.L + pos;
    if (a.p_tok) a.p_tok[o] = NAN;
    if (a.q_tok) a.q_tok[o] = NAN;
    if (a.f) a.f[o] = NAN;
  }
  if (w >= 0 && lane == w) a.seq_stat[b] = make_float4(Ct, St, Cd, Sd);      // position tau, or the bonus row
  if (lane == 0) {
    a.tau_ws[b] = w >= 0 ? lo + w : -1;
    if (w >= 0) a.accept_len[b] = lo + w;
  }
}

// Chunk masses of the sampled rows as a launch of its own (the three-launch form: rows of more than
// 64 statistics chunks, draft windows beyond kTauRows positions, the stand-alone resampling call).
template <int DT, bool XF, bool AL, int kT, bool LAN>
__global__ __launch_bounds__(kThreads) void sequence_masses_kernel(const KArgs a) {
  constexpr int kE = Vec<DT>::kE;
  constexpr int kChunk2 = kT * kThreads * kE;            // logits per sampling chunk
  __shared__ Smem sm;
  const int C = a.nchunks;
  const int b = blockIdx.x / C, c = blockIdx.x - b * C;
  const int tau = a.resample_only ? 0 : a.accept_len[b];
  const SampledRow r = sampled_row<DT, XF>(a, b, tau);
  if (r.none) return;
  // left by accept_kernel: the same for every thread, read straight from the workspace (a scalar
  // load that is in flight while the chunk's vector loads are issued)
  const float4 rs = sampled_row_stats(a, b, r, &sm.rowstat);
  // the mass pass reads every chunk of the row exactly once: nontemporal loads
  constexpr int kA = AL ? kAlignedStream : kUnaligned;
  const int64_t base = int64_t(c) * kChunk2;
  RowRegs<DT, XF, kT> rt, rd;
  load_chunk<DT, XF, kA, kT>(rt, r.t_c, r.t_u, base, a.V, a.cfg_scale, a.inv_T, r.thr_t);
  if (!r.bonus) load_chunk<DT, XF, kA, kT>(rd, r.d_c, r.d_u, base, a.V, a.cfg_scale, a.inv_T, r.thr_d);
  else rd.clear();                                    // never read in mode P
  const ResidCoef k{rs.x, 1.f / rs.y, rs.z, r.bonus ? 1.f : 1.f / rs.w, r.omega,
                    r.bonus ? kModeP : (a.resample_mode == 1 ? kModeVanilla : kModeOpt)};
  // Eq. g_lantern: this thread's part of the patch
  LanPatch lp{0u, -1, 1.f};
  if constexpr (LAN) {
    if (!r.bonus) lp = lan_patch_tile<Vec<DT>::kE>(a, b, r.j, r.omega, base, kChunk2);
  }
  // only the chunk's total is needed: per-thread sum in ascending tile order, one wave reduction,
  // one barrier
  float acc = 0.f;
#pragma unroll
  for (int t = 0; t < kT; ++t) {
#pragma unroll
    for (int e = 0; e < kE; ++e) acc = __fadd_rn(acc, tile_elem<DT, XF, kT, LAN>(rt, rd, k, lp, t, e));
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) sm.scan_tot[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0)
    a.chunk_R[int64_t(b) * C + c] = __fadd_rn(__fadd_rn(sm.scan_tot[0], sm.scan_tot[1]), __fadd_rn(sm.scan_tot[2], sm.scan_tot[3]));
}

template <int DT, bool XF, bool AL, bool LAN>
__global__ __launch_bounds__(kThreadsW) void sequence_select_kernel(const KArgs a) {
  constexpr int kE = Vec<DT>::kE;
  constexpr int kChunk2 = kChunk / 2;                     // logits per sampling chunk (8192)
  constexpr int kVS = kChunk2 / (kThreadsW * kE);         // consecutive vectors per thread: 1 (bf16) / 2 (fp32)
  __shared__ SmemW sm;
  __shared__ float cm[kStage];
  __shared__ ExactSmem<kThreadsW> smx;
  const int C = a.nchunks;
  const int b = blockIdx.x;
  if (threadIdx.x == 0) sm.needs64 = 0;           // barriers lie between this and its readers
  // what does not depend on tau is requested before tau arrives: lane c's chunk mass (rows of up
  // to 64 chunks) and the uniform
  const int lane0 = threadIdx.x & 63;
  float m_early = (C <= 64 && lane0 < C) ? a.chunk_R[int64_t(b) * C + lane0] : 0.f;
  float u_early = a.u_res[b];
  asm volatile("" : "+v"(m_early), "+v"(u_early));
  const SampledRow r = sampled_row<DT, XF>(a, b, a.resample_only ? 0 : a.accept_len[b]);
  if (r.none) {
    if (threadIdx.x == 0) {
      a.next_token[b] = -1;
      if (a.resid_mass) a.resid_mass[b] = 0.f;
    }
    return;
  }
  const float4 rs = sampled_row_stats(a, b, r, &sm.rowstat);
  ResidCoef k{rs.x, 1.f / rs.y, rs.z, r.bonus ? 1.f : 1.f / rs.w, r.omega,
              r.bonus ? kModeP : (a.resample_mode == 1 ? kModeVanilla : kModeOpt)};
  const int law = k.mode;                                 // before any fall-back to p

  // mass of chunk cc under the fallback law p, from the chunk statistics of the statistics pass
  const int per = kChunk2 / a.chunk1;
  auto p_mass = [&](int cc) -> float {
    float m = 0.f;
    for (int q = cc * per; q < min((cc + 1) * per, a.c1); ++q) {
      const float2 pp = a.part[int64_t(r.rt_) * a.c1 + q];
      m = __fadd_rn(m, __fmul_rn(__fmul_rn(pp.y, exp2_fast(pp.x - rs.x)), k.at));
    }
    return m;
  };
  // The chunk that holds u*R: first with positive mass whose inclusive sum exceeds u*R, else the
  // last with mass.  chunk_trust: no fall-back at this level, and the law is heavy enough for its
  // fp32 mass to be accurate.
  float R, cbase = 0.f;
  int cs = -1;
  bool fallback = false, chunk_trust = true;
  if (C <= 64) {
    // up to 64 chunks (rows of 524288 logits): lane c of every wave takes chunk c, one memory
    // round trip and a wave scan, no LDS and no barrier; every wave gets the same answer
    const int lane = threadIdx.x & 63;
    float m = m_early;
    float incl = wave_scan_incl(m);
    R = lane_f(incl, 63);
    if (!(R > 0.f)) {    // no rejection possible at this position: any law is optimal, use p
      fallback = true;
      k.mode = kModeP;
      m = lane < C ? p_mass(lane) : 0.f;
      incl = wave_scan_incl(m);
      R = lane_f(incl, 63);
    }
    const float v = __fmul_rn(u_early, R);
    const float excl = wave_prev_lane(incl);
    const bool pos = m > 0.f;
    const unsigned long long bh = __ballot(pos && incl > v), bp = __ballot(pos);
    chunk_trust = bh != 0;
    cs = bh ? __ffsll((long long)bh) - 1 : (bp ? 63 - __clzll((long long)bp) : 0);
    cbase = lane_f(excl, cs);
  } else {
    // longer rows: chunk masses staged in LDS by all threads (one latency), then walked in
    // ascending order by every thread for itself; more than kStage chunks walk global memory
    const bool staged = C <= kStage;
    auto chunk_mass = [&](int cc) -> float {
      if (staged) return cm[cc];
      return fallback ? p_mass(cc) : a.chunk_R[int64_t(b) * C + cc];
    };
    if (staged) {
      for (int cc = threadIdx.x; cc < C; cc += kThreadsW) cm[cc] = a.chunk_R[int64_t(b) * C + cc];
      __syncthreads();
    }
    R = 0.f;
    for (int cc = 0; cc < C; ++cc) R = __fadd_rn(R, chunk_mass(cc));
    if (!(R > 0.f)) {
      fallback = true;
      k.mode = kModeP;
      if (staged) {
        __syncthreads();
        for (int cc = threadIdx.x; cc < C; cc += kThreadsW) cm[cc] = p_mass(cc);
        __syncthreads();
      }
      R = 0.f;
      for (int cc = 0; cc < C; ++cc) R = __fadd_rn(R, chunk_mass(cc));
    }
    const float v = __fmul_rn(a.u_res[b], R);
    int clast = -1;
    float cbase_last = 0.f, cum = 0.f;
    for (int cc = 0; cc < C; ++cc) {
      const float m = chunk_mass(cc);
      if (m > 0.f) {
        if (cs < 0 && __fadd_rn(cum, m) > v) { cs = cc; cbase = cum; }
        clast = cc; cbase_last = cum;
      }
      cum = __fadd_rn(cum, m);
    }
    chunk_trust = cs >= 0;
    if (cs < 0) { cs = clast; cbase = cbase_last; }
    if (cs < 0) cs = 0;
  }
  chunk_trust = chunk_trust && !fallback && (law == kModeP || R >= kSafeMass);
  const float v_in = __fsub_rn(__fmul_rn(a.u_res[b], R), cbase);   // mass left to walk inside the chunk

  // the chosen chunk, thread t holding its vectors t*kVS ..: same search as on short rows, for
  // the mass that is left to walk inside the chunk
  const int64_t base = int64_t(cs) * kChunk2;
  RowRegs<DT, XF, kVS> rt, rd;
  load_chunk<DT, XF, AL, kVS, 1, kVS>(rt, r.t_c, r.t_u, base, a.V, a.cfg_scale, a.inv_T, r.thr_t);
  if (!r.bonus) load_chunk<DT, XF, AL, kVS, 1, kVS>(rd, r.d_c, r.d_u, base, a.V, a.cfg_scale, a.inv_T, r.thr_d);
  else rd.clear();                                    // never read in mode P
  LanPatch lp{0u, -1, 1.f};
  if constexpr (LAN) {
    if (!r.bonus && !fallback) lp = lan_patch_span(a, b, r.j, r.omega, base + int64_t(threadIdx.x) * (kVS * kE), kVS * kE);
  }
  float R_chunk;
  bool writer, trust;
  int token = (int)base + sample_whole<DT, XF, kVS, LAN, true>(rt, rd, k, v_in, a.V - (int)base, sm, R_chunk, writer, trust,
                                                               lp);
  if (draw_needs_fp64(writer, trust && chunk_trust, a.exact_draw, &sm.needs64)) {
    ExactJob job{{r.t_c, r.t_u, r.thr_t, (double)rs.x}, {r.d_c, r.d_u, r.thr_d, (double)rs.z}, DT, XF, a.V, a.cfg_scale,
                 a.inv_T, r.omega, law, nullptr, 0, 0, 0};
    if constexpr (LAN) {
      if (!r.bonus) {
        job.lan_x = min(max(a.tokens[int64_t(b) * a.L + r.j], 0), a.V - 1);
        job.nbr_row = a.nbr + int64_t(job.lan_x) * a.lan_k;
        job.lan_k = a.lan_k;
        job.lan_m = a.lan_count[int64_t(b) * a.L + r.j];
      }
    }
    token = exact_draw<kThreadsW>(job, a.u_res[b], R, smx);
    writer = threadIdx.x == 0;
  }
  if (writer) {
    a.next_token[b] = token;
    if (a.resid_mass) a.resid_mass[b] = R;
  }
}

// ============================================================================ long rows, one launch
// Everything after the statistics pass for sequences whose rows have at most 64 statistics chunks
// and at most kTauRows positions: G workgroups of 256 threads per sequence.
//   1. every workgroup finds tau for itself from the chunk statistics (find_tau_from_parts; the
//      first one writes accept_len and the per-position outputs);
//   2. workgroup g streams chunks g, g + G, ... of the sampled row pair (8192 logits each, at most
//      kTailPer per workgroup) and leaves each chunk's residual mass in the workspace;
//   3. it then takes a ticket of its sequence; the workgroup that draws the last ticket knows that
//      all chunk masses of the sequence are written: it picks the chunk that holds u*R (lane per
//      chunk, one wave scan), re-reads that one chunk and finds the token in it, tile -> thread ->
//      element, like the early-exit kernel does on its rows.
// No workgroup waits for another: whoever comes last does the rest, so the grid need not be
// resident at once.  Ordering: a chunk mass is written with a device-scope atomic store whose
// completion the writer awaits before its device-scope fetch-add on the ticket, and the last
// workgroup reads the masses with device-scope atomic loads.  The tickets are cleared by the
// statistics launch of the same call (first workgroup of every sequence).
// Against the three launches this replaces (accept_kernel, sequence_masses_kernel,
// sequence_select_kernel) it saves two launch gaps and one of the three latency chains.
constexpr int kTailPer = 8;      // chunks one workgroup of the tail launch takes at most
template <int DT, bool XF, bool AL, int kT, bool LAN>
__global__ __launch_bounds__(kThreads) void sequence_tail_kernel(const KArgs a) {
  constexpr int kE = Vec<DT>::kE;
  constexpr int kChunk2 = kT * kThreads * kE;            // logits per sampling chunk (8192)
  __shared__ Smem sm;
  __shared__ SmemTau smt;
  __shared__ ExactSmem<kThreads> smx;
  __shared__ int last_flag;
  const int C = a.nchunks, G = a.tail_groups;
  const int b = blockIdx.x / G, g = blockIdx.x - b * G;
  const int tau = find_tau_from_parts(a, b, g == 0, smt);
  const float4 rs = smt.rowstat;                         // statistics of the sampled row
  const SampledRow r = sampled_row<DT, XF>(a, b, tau, smt.omega);
  if (r.none) {
    if (g == 0 && threadIdx.x == 0) {
      a.next_token[b] = -1;
      if (a.resid_mass) a.resid_mass[b] = 0.f;
    }
    return;
  }
  ResidCoef k{rs.x, 1.f / rs.y, rs.z, r.bonus ? 1.f : 1.f / rs.w, r.omega,
              r.bonus ? kModeP : (a.resample_mode == 1 ? kModeVanilla : kModeOpt)};
  const int law = k.mode;
  // The mass pass: this workgroup's chunks g, g + G, ... (at most kTailPer of them), each read
  // exactly once (nontemporal loads).  Two register sets alternate, so the loads of the next chunk
  // are in flight while the current one is summed; a thread keeps one partial sum per chunk and
  // nothing is exchanged between threads until all chunks are done (no barrier in the loop).
  constexpr int kA = AL ? kAlignedStream : kUnaligned;
  float acc[kTailPer];
#pragma unroll
  for (int i = 0; i < kTailPer; ++i) acc[i] = 0.f;
  auto fetch = [&](RowRegs<DT, XF, kT>& rt, RowRegs<DT, XF, kT>& rd, int c) {
    const int64_t base = int64_t(c) * kChunk2;
    load_chunk<DT, XF, kA, kT>(rt, r.t_c, r.t_u, base, a.V, a.cfg_scale, a.inv_T, r.thr_t);
    if (!r.bonus) load_chunk<DT, XF, kA, kT>(rd, r.d_c, r.d_u, base, a.V, a.cfg_scale, a.inv_T, r.thr_d);
    else rd.clear();                                    // never read in mode P
  };
  auto chunk_sum = [&](const RowRegs<DT, XF, kT>& rt, const RowRegs<DT, XF, kT>& rd, int c) -> float {
    LanPatch lp{0u, -1, 1.f};
    if constexpr (LAN) {
      if (!r.bonus) lp = lan_patch_tile<kE>(a, b, r.j, r.omega, int64_t(c) * kChunk2, kChunk2);
    }
    float sum = 0.f;
#pragma unroll
    for (int t = 0; t < kT; ++t) {
#pragma unroll
      for (int e = 0; e < kE; ++e) sum = __fadd_rn(sum, tile_elem<DT, XF, kT, LAN>(rt, rd, k, lp, t, e));
    }
    return sum;
  };
  {
    RowRegs<DT, XF, kT> rt0, rd0, rt1, rd1;
    if (g < C) fetch(rt0, rd0, g);
#pragma unroll
    for (int i = 0; i < kTailPer; i += 2) {
      const int c0 = g + i * G, c1 = c0 + G, c2 = c1 + G;
      if (c1 < C) fetch(rt1, rd1, c1);
      if (c0 < C) acc[i] = chunk_sum(rt0, rd0, c0);
      if (i + 2 < kTailPer && c2 < C) fetch(rt0, rd0, c2);
      if (i + 1 < kTailPer && c1 < C) acc[i + 1] = chunk_sum(rt1, rd1, c1);
    }
  }
  // one reduction for all chunks of this workgroup: wave sums to LDS, then thread i adds the four
  // wave sums of its i-th chunk and writes the chunk's mass with a device-scope store
#pragma unroll
  for (int i = 0; i < kTailPer; ++i) {
    const float ws = wave_sum(acc[i]);
    if ((threadIdx.x & 63) == 0) sm.tile_part[threadIdx.x >> 6][i] = ws;
  }
  __syncthreads();
  if ((int)threadIdx.x < kTailPer && g + (int)threadIdx.x * G < C) {
    const int i = threadIdx.x;
    const float m = __fadd_rn(__fadd_rn(sm.tile_part[0][i], sm.tile_part[1][i]), __fadd_rn(sm.tile_part[2][i], sm.tile_part[3][i]));
    __hip_atomic_store(&a.chunk_R[int64_t(b) * C + g + i * G], m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // this thread's store has been acknowledged before the barrier that precedes the ticket
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  __syncthreads();
  // the ticket: this workgroup's masses were written with device-scope stores, which go through to
  // the point where every compute die sees them, and each writer has waited for the acknowledgement
  // before the barrier above; only then does the workgroup count itself.  (A release fence would do the same and more: it also
  // writes back every dirty line of the die's L2, which costs far more than this launch.)
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(&a.ticket[b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    last_flag = old == G - 1;
  }
  __syncthreads();
  if (!last_flag) return;
  // the last workgroup reads the masses with device-scope loads (never from a stale cache line)

  // the chunk that holds u*R: first with positive mass whose inclusive sum exceeds u*R, else the
  // last with mass; lane c of every wave takes chunk c (C <= 64)
  const int lane = threadIdx.x & 63;
  const int per = kChunk2 / a.chunk1;
  auto p_mass = [&](int cc) -> float {        // mass of chunk cc under the fall-back law p, from the statistics pass
    float m = 0.f;
    for (int q = cc * per; q < min((cc + 1) * per, a.c1); ++q) {
      const float2 pp = a.part[int64_t(r.rt_) * a.c1 + q];
      m = __fadd_rn(m, __fmul_rn(__fmul_rn(pp.y, exp2_fast(pp.x - rs.x)), k.at));
    }
    return m;
  };
  float m = lane < C ? __hip_atomic_load(&a.chunk_R[int64_t(b) * C + lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
  float incl = wave_scan_incl(m);
  float R = lane_f(incl, 63);
  bool fallback = false;
  if (!(R > 0.f)) {    // no rejection possible at this position: any law is optimal, use p
    fallback = true;
    k.mode = kModeP;
    m = lane < C ? p_mass(lane) : 0.f;
    incl = wave_scan_incl(m);
    R = lane_f(incl, 63);
  }
  const float v = __fmul_rn(a.u_res[b], R);
  const float excl = wave_prev_lane(incl);
  const bool pos = m > 0.f;
  const unsigned long long bh = __ballot(pos && incl > v), bp = __ballot(pos);
  const int cs = bh ? __ffsll((long long)bh) - 1 : (bp ? 63 - __clzll((long long)bp) : 0);
  const float v_in = __fsub_rn(v, lane_f(excl, cs));   // mass left to walk inside the chunk
  bool trust = bh != 0 && !fallback && (law == kModeP || R >= kSafeMass);

  const int64_t base = int64_t(cs) * kChunk2;
  RowRegs<DT, XF, kT> rt, rd;
  load_chunk<DT, XF, AL ? kAligned : kUnaligned, kT>(rt, r.t_c, r.t_u, base, a.V, a.cfg_scale, a.inv_T, r.thr_t);
  if (!r.bonus) load_chunk<DT, XF, AL ? kAligned : kUnaligned, kT>(rd, r.d_c, r.d_u, base, a.V, a.cfg_scale, a.inv_T, r.thr_d);
  else rd.clear();
  LanPatch lp{0u, -1, 1.f};
  if constexpr (LAN) {
    if (!r.bonus && !fallback) lp = lan_patch_tile<kE>(a, b, r.j, r.omega, base, kChunk2);
  }
  float part[kT];
  chunk_masses<DT, XF, kT, LAN>(rt, rd, k, part, sm, lp);
  bool chunk_trust;
  int token = (int)base + max(chunk_select<DT, XF, kT, LAN>(rt, rd, k, part, v_in, sm, chunk_trust, lp), 0);
  token = min(token, a.V - 1);
  if (!(trust && chunk_trust) || a.exact_draw) {
    ExactJob job{{r.t_c, r.t_u, r.thr_t, (double)rs.x}, {r.d_c, r.d_u, r.thr_d, (double)rs.z}, DT, XF, a.V, a.cfg_scale,
                 a.inv_T, r.omega, law, nullptr, 0, 0, 0};
    if constexpr (LAN) {
      if (!r.bonus) {
        job.lan_x = min(max(a.tokens[int64_t(b) * a.L + r.j], 0), a.V - 1);
        job.nbr_row = a.nbr + int64_t(job.lan_x) * a.lan_k;
        job.lan_k = a.lan_k;
        job.lan_m = a.lan_count[int64_t(b) * a.L + r.j];
      }
    }
    token = exact_draw<kThreads>(job, a.u_res[b], R, smx);
  }
  if (threadIdx.x == 0) {
    a.next_token[b] = token;
    if (a.resid_mass) a.resid_mass[b] = R;
  }
}

}  // namespace csd
