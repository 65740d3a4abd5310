// Second launch of a verify call on rows of at most 16384 logits: sequence_whole_kernel with its
// register-resident sampler; the stand-alone neighbour aggregation kernel.
#pragma once
#include "exact_draw.h"
#include "sequence_common.h"
#include "stats_kernels.h"

namespace csd {

// ============================================================================ kernel 2, rows of one chunk
// One workgroup of 1024 threads per sequence (rows of at most 16384 logits): find tau, re-read
// the one row pair that is sampled from, and draw x_{tau+1} (Eq. opt_G / Eq. g_tsd / p_{L+1}).
// This kernel is a latency chain, not a bandwidth kernel, so it is laid out for few dependent
// steps: thread t owns the kVW CONSECUTIVE 16-byte vectors t*kVW .. t*kVW+kVW-1 of the row, so
// the running mass in ascending token order is simply a prefix sum over threads.  Per thread:
// one partial mass per vector; block-wide: one scan.  The thread whose interval contains u*R
// finds the vector among its partials and re-evaluates that vector's elements.

// One draw from the resampling law of a row pair that 1024 threads hold in registers (thread t
// owns the kVW consecutive vectors t*kVW ..): per-vector masses, one block scan, then vector and
// element inside the thread whose interval contains u*R.  If the law has no mass (no rejection
// is possible at this position) it falls back to p.  The token is returned in ONE thread, the one
// that found it (writer = true there), so that no barrier is spent on handing it around; R, the
// law's mass, is known to every thread.
// ABS: `u` is not the uniform but the mass to walk itself (the caller has taken u*R of a longer
// row and subtracted what lies before this part of it); V is then the number of tokens from the
// first one held here to the end of the row.
// trust (meaningful in the writer thread only): the fp32 result stands -- no level of the search
// had to fall back to its last entry with mass and (not ABS, where the caller knows the whole
// law's mass) the law weighs at least kSafeMass.  Otherwise the caller re-does the draw in fp64
// (exact_draw.h).
template <int DT, bool XF, int kVW, bool LAN = false, bool ABS = false>
__device__ __forceinline__ int sample_whole(const RowRegs<DT, XF, kVW>& rt, const RowRegs<DT, XF, kVW>& rd,
                                            ResidCoef k, float u, int V, SmemW& sm, float& R, bool& writer,
                                            bool& trust, const LanPatch lp = LanPatch{0u, -1, 1.f}) {
  constexpr int kE = Vec<DT>::kE;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  // mass of element e of this thread's vector v
  auto relem = [&](int v, int e) -> float {
    if constexpr (LAN) return resid_elem_lan(rt.get(v, e), rd.get(v, e), k, lp, v * kE + e);
    else return resid_elem(rt.get(v, e), rd.get(v, e), k);
  };
  float r[kVW * kE];           // masses of this thread's tokens, kept for the final search
  float part[kVW], mine, incl, excl;
  R = 0.f;
  bool fell_back = false;      // the law had no fp32 mass and p took its place
  for (int attempt = 0; attempt < 2; ++attempt) {
    mine = 0.f;
#pragma unroll
    for (int v = 0; v < kVW; ++v) {
      float acc = 0.f;
#pragma unroll
      for (int e = 0; e < kE; ++e) {
        r[v * kE + e] = relem(v, e);
        acc = __fadd_rn(acc, r[v * kE + e]);
      }
      part[v] = acc;
      mine = __fadd_rn(mine, acc);
    }
    const float incl_w = wave_scan_incl(mine);
    const float excl_w = wave_prev_lane(incl_w);
    __syncthreads();                                  // earlier readers of scan_tot are done
    if (lane == 63) sm.scan_tot[wv] = incl_w;
    __syncthreads();
    // every wave scans the 16 wave totals for itself (one LDS read per lane, one row of DPP
    // shifts): its own offset is the exclusive value at lane wv, R the inclusive value at lane 15
    static_assert(kWavesW == 16, "one DPP row holds the wave totals");
    float tot = lane < kWavesW ? sm.scan_tot[lane] : 0.f;
    tot = __fadd_rn(tot, dpp_f<kDppRowShr1>(tot));
    tot = __fadd_rn(tot, dpp_f<kDppRowShr2>(tot));
    tot = __fadd_rn(tot, dpp_f<kDppRowShr4>(tot));
    tot = __fadd_rn(tot, dpp_f<kDppRowShr8>(tot));
    R = lane_f(tot, kWavesW - 1);
    const float woff = wv == 0 ? 0.f : lane_f(tot, wv - 1);
    incl = __fadd_rn(woff, incl_w);
    excl = __fadd_rn(woff, excl_w);
    if (__builtin_expect(R > 0.f || k.mode == kModeP, 1)) break;
    k.mode = kModeP;   // no rejection possible at this position: any law is optimal, use p
    fell_back = true;
  }

  // thread: first with positive mass whose inclusive sum exceeds u*R, else the last with mass
  const float v = ABS ? u : __fmul_rn(u, R);
  const bool pos = mine > 0.f;
  const bool hit = pos && (incl > v);
  const unsigned long long bh = __ballot(hit), bp = __ballot(pos);
  if (lane == 0) {
    sm.pick[wv] = bh ? (wv * 64 + __ffsll((long long)bh) - 1) : 0x7fffffff;
    sm.pick_last[wv] = bp ? (wv * 64 + 63 - __clzll((long long)bp)) : -1;
  }
  __syncthreads();
  int win = 0x7fffffff, last_pos = -1;
#pragma unroll
  for (int w = 0; w < kWavesW; ++w) { win = min(win, sm.pick[w]); last_pos = max(last_pos, sm.pick_last[w]); }
  const bool thread_fallback = win == 0x7fffffff;
  if (thread_fallback) win = last_pos;
  writer = win >= 0 ? (int)threadIdx.x == win : threadIdx.x == 0;   // a row without any mass: token 0
  trust = true;
  int token = 0;
  if ((int)threadIdx.x == win) {
    // vector, then element: same rule at each level
    const float v2 = v - excl;
    int vs = -1, vlast = 0;
    float vbase = 0.f, vbase_last = 0.f, cum = 0.f;
#pragma unroll
    for (int q = 0; q < kVW; ++q) {
      if (part[q] > 0.f) {
        if (vs < 0 && __fadd_rn(cum, part[q]) > v2) { vs = q; vbase = cum; }
        vlast = q; vbase_last = cum;
      }
      cum = __fadd_rn(cum, part[q]);
    }
    const bool vector_fallback = vs < 0;
    if (vector_fallback) { vs = vlast; vbase = vbase_last; }
    const float v3 = v2 - vbase;
    float rv[kE];                 // the selected vector's masses
#pragma unroll
    for (int e = 0; e < kE; ++e) {
      rv[e] = r[e];
#pragma unroll
      for (int q = 1; q < kVW; ++q) rv[e] = (q == vs) ? r[q * kE + e] : rv[e];
    }
    int found = -1, last = 0;
    float run = 0.f;
#pragma unroll
    for (int e = 0; e < kE; ++e) {
      if (rv[e] > 0.f) {
        last = e;
        run = __fadd_rn(run, rv[e]);
        if (found < 0 && run > v3) found = e;
      }
    }
    const bool element_fallback = found < 0;
    if (element_fallback) found = last;
    token = (win * kVW + vs) * kE + found;
    trust = !(thread_fallback || vector_fallback || element_fallback || fell_back) &&
            (ABS || k.mode == kModeP || R >= kSafeMass);
  } else if (writer) {
    trust = !fell_back;        // no mass at all: a row without a finite logit, outside the contract
  }
  return token >= V ? V - 1 : token;
}

// After a draw: the whole workgroup learns whether the thread that found the token trusts it.
// `flag` is an LDS word that thread 0 cleared before an earlier barrier.
__device__ __forceinline__ bool draw_needs_fp64(bool writer, bool trust, int force, int* flag) {
  if (writer && !trust) *flag = 1;
  __syncthreads();
  return *flag != 0 || force != 0;
}

// MUL = 2: the same for rows of up to 32768 logits, whose pair still fits the registers of 1024
// threads (32 words per row and thread) -- one launch where the long-row form needs three.  (Four
// times the row, 65536 packed bf16 logits, was measured too: it spills and is slower than the
// three launches.)
template <int DT, bool XF, bool AL, bool LAN, int MUL = 1>
__global__ __launch_bounds__(kThreadsW) void sequence_whole_kernel(const KArgs a) {
  constexpr int kE = Vec<DT>::kE, kES = Vec<DT>::kES;
  constexpr int kVW = MUL * kChunk / (kThreadsW * kE);   // vectors per thread: MUL * 2 (bf16) / MUL * 4 (fp32)
  static_assert(MUL == 1 || (MUL == 2 && !LAN), "the neighbour patch is one 32-bit mask per thread");
  static_assert((RowRegs<DT, XF, kVW>::kRaw ? kVW * 4 : kVW * kE) <= 32, "a row pair must fit the registers");
  __shared__ SmemW sm;
  __shared__ ExactSmem<kThreadsW> smx;
  const int b = blockIdx.x;
  const int rps = a.L + a.has_bonus;
  const bool masked = XF && a.top_k > 0;
  if (threadIdx.x == 0) sm.needs64 = 0;           // several barriers lie between this and its readers

  int j = 0;
  if (!a.resample_only) {
    j = find_tau<DT, XF, kThreadsW>(a, b, true, sm.pick, &sm.rowstat);
    if (j >= a.L && !a.has_bonus) {
      if (threadIdx.x == 0) {
        a.next_token[b] = -1;
        if (a.resid_mass) a.resid_mass[b] = 0.f;
      }
      return;
    }
  }
  const bool bonus = a.resample_only ? (a.d == nullptr) : (j == a.L);
  const int rt_ = b * rps + j, rd_ = a.rows_t + b * a.L + j;
  if (a.resample_only) {
    if (threadIdx.x == 0) {
      float Ct, St, Cd = kRefFloor, Sd = 0.f;
      combine_row(a, rt_, Ct, St);
      if (!bonus) combine_row(a, rd_, Cd, Sd);
      sm.rowstat = make_float4(Ct, St, Cd, Sd);
    }
    __syncthreads();
  }
  const float4 rs = sm.rowstat;
  const char* t_c = row_ptr(a.t, int64_t(b) * a.t_sb + int64_t(j) * a.t_sl, kES);
  const char* t_u = row_ptr(a.tu, int64_t(b) * a.t_sb + int64_t(j) * a.t_sl, kES);
  const char* d_c = bonus ? nullptr : row_ptr(a.d, int64_t(b) * a.d_sb + int64_t(j) * a.d_sl, kES);
  const char* d_u = bonus ? nullptr : row_ptr(a.du, int64_t(b) * a.d_sb + int64_t(j) * a.d_sl, kES);
  const float thr_t = masked ? a.thr[rt_] : -INFINITY;
  const float thr_d = (masked && !bonus) ? a.thr[rd_] : -INFINITY;
  const float omega = bonus ? 1.f : a.omega[int64_t(b) * a.om_sb + j];
  ResidCoef k{rs.x, 1.f / rs.y, rs.z, bonus ? 1.f : 1.f / rs.w, omega,
              bonus ? kModeP : (a.resample_mode == 1 ? kModeVanilla : kModeOpt)};

  RowRegs<DT, XF, kVW> rt, rd;
  load_chunk<DT, XF, AL, kVW, 1, kVW>(rt, t_c, t_u, 0, a.V, a.cfg_scale, a.inv_T, thr_t);
  if (!bonus) load_chunk<DT, XF, AL, kVW, 1, kVW>(rd, d_c, d_u, 0, a.V, a.cfg_scale, a.inv_T, thr_d);
  else rd.clear();                                    // never read in mode P

  float R;
  int token;
  bool writer, trust;
  ExactJob job{{t_c, t_u, thr_t, (double)rs.x}, {d_c, d_u, thr_d, (double)rs.z}, DT, XF, a.V, a.cfg_scale, a.inv_T,
               omega, k.mode, nullptr, 0, 0, 0};
  if constexpr (LAN) {
    // Eq. g_lantern: the law is [P^{k,lambda} - q]_+ around the rejected token x~_j; this thread
    // owns the kVW*kE consecutive tokens from first_tok on
    LanPatch lp{0u, -1, 1.f};
    if (!bonus) {
      k.mode = kModeVanilla;
      const int first_tok = threadIdx.x * (kVW * kE);
      const int xd = min(max(a.tokens[int64_t(b) * a.L + j], 0), a.V - 1);
      const int m = a.lan_count[int64_t(b) * a.L + j];
      lp.agg = omega;                                   // sum over the set / p(x~_j), from lantern_agg_position
      const int dx = xd - first_tok;
      if (dx >= 0 && dx < kVW * kE) lp.aggpos = dx;
      const int32_t* row = a.nbr + int64_t(xd) * a.lan_k;
      int taken = 0;
      for (int jj = 0; jj < a.lan_k && taken < m; ++jj) {   // the first m valid neighbours are the members
        const int n = row[jj];
        if (n < 0 || n >= a.V || n == xd) continue;
        ++taken;
        const int dn = n - first_tok;
        if (dn >= 0 && dn < kVW * kE) lp.zmask |= 1u << dn;
      }
      job.mode = kModeVanilla;
      job.nbr_row = row; job.lan_k = a.lan_k; job.lan_m = m; job.lan_x = xd;
    }
    token = sample_whole<DT, XF, kVW, true>(rt, rd, k, a.u_res[b], a.V, sm, R, writer, trust, lp);
  } else {
    token = sample_whole<DT, XF, kVW>(rt, rd, k, a.u_res[b], a.V, sm, R, writer, trust);
  }
  if (__builtin_expect(draw_needs_fp64(writer, trust, a.exact_draw, &sm.needs64), 0)) {     // rare: keep its code off the hot path
    token = exact_draw<kThreadsW>(job, a.u_res[b], R, smx);
    writer = threadIdx.x == 0;
  }
  if (writer) {
    a.next_token[b] = token;
    if (a.resid_mass) a.resid_mass[b] = R;
  }
}

}  // namespace csd
