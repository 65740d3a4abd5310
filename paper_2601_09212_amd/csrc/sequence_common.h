// Pieces shared by the per-sequence kernels: combining chunk statistics, the residual law
// element by element, chunk masses and selection, the accept test (eval_position, find_tau).
#pragma once
#include "kernel_common.h"

namespace csd {


// Optional middle kernel (rows with more than kMaxDirect statistics chunks): one wave per row
// combines the row's chunk statistics into one (reference exponent, sum) pair.  Lanes take
// chunks cc = lane, lane+64, ...; the reference is the maximum, sums are rescaled by exact
// powers of two and added in a fixed order.
__device__ __forceinline__ void combine_row_wave(const KArgs& a, int r) {
  const int lane = threadIdx.x & 63;
  const float2* p = a.part + int64_t(r) * a.c1;
  float m = kRefFloor;
  for (int cc = lane; cc < a.c1; cc += 64) m = fmaxf(m, p[cc].x);
  m = wave_max(m);
  float s = 0.f;
  for (int cc = lane; cc < a.c1; cc += 64) s = __fadd_rn(s, p[cc].y * exp2_fast(p[cc].x - m));
  s = wave_sum(s);
  if (lane == 0) a.rowstat[r] = make_float2(m, s);
}

// Statistics of row r from at most kMaxDirect entries (a.stat, a.cs entries per row), all
// loaded before any is used: reference = max, sum rescaled by exact powers of two.
constexpr int kMaxDirect = 4;
constexpr int kStage = 1024;   // chunk masses staged in LDS by the sampling kernel
// In two halves, for callers that want the loads of several rows in flight before anything waits
// for the first of them.
__device__ __forceinline__ void load_row_parts(const KArgs& a, int r, float2 (&v)[kMaxDirect]) {
  const float2* p = a.stat + int64_t(r) * a.cs;
#pragma unroll
  for (int cc = 0; cc < kMaxDirect; ++cc) v[cc] = p[cc < a.cs ? cc : 0];
}
__device__ __forceinline__ void combine_parts(const KArgs& a, float2 (&v)[kMaxDirect], float& C, float& S) {
#pragma unroll
  for (int cc = 0; cc < kMaxDirect; ++cc)
    if (cc >= a.cs) v[cc] = make_float2(kRefFloor, 0.f);
  float m = kRefFloor;
#pragma unroll
  for (int cc = 0; cc < kMaxDirect; ++cc) m = fmaxf(m, v[cc].x);
  float s = 0.f;
#pragma unroll
  for (int cc = 0; cc < kMaxDirect; ++cc) s = __fadd_rn(s, v[cc].y * exp2_fast(v[cc].x - m));
  C = m; S = s;
}
__device__ __forceinline__ void combine_row(const KArgs& a, int r, float& C, float& S) {
  float2 v[kMaxDirect];
  load_row_parts(a, r, v);
  combine_parts(a, v, C, S);
}

// Unnormalised resampling mass of one token.  p = 2^(lt*log2e - Ct) / St etc.
struct ResidCoef {
  float Ct, at, Cd, ad, omega;
  int mode;
};
__device__ __forceinline__ float resid_elem(float lt, float ld, const ResidCoef& k) {
  const float p = __fmul_rn(exp2_fast(__fmaf_rn(lt, kLog2e, -k.Ct)), k.at);
  if (k.mode == kModeP) return p;
  const float q = __fmul_rn(exp2_fast(__fmaf_rn(ld, kLog2e, -k.Cd)), k.ad);
  const float qf = (k.mode == kModeOpt) ? fminf(q, __fmul_rn(k.omega, p)) : q;
  return fmaxf(__fsub_rn(p, qf), 0.f);
}

// Eq. p_lantern as a patch of the target row held by one thread: the members of the rejected
// token's neighbour set lose their probability (bit n of zmask: this thread's element n is a
// member) and the rejected token itself carries the aggregated one (p times agg).
struct LanPatch {
  uint32_t zmask;
  int aggpos;       // this thread's element that is the rejected token, or -1
  float agg;
};
// Unnormalised mass [P^{k,lambda} - q]_+ (Eq. g_lantern) of this thread's element n.
__device__ __forceinline__ float resid_elem_lan(float lt, float ld, const ResidCoef& k, const LanPatch& lp, int n) {
  float p = __fmul_rn(exp2_fast(__fmaf_rn(lt, kLog2e, -k.Ct)), k.at);
  if (k.mode == kModeP) return p;
  p = ((lp.zmask >> n) & 1u) ? 0.f : p;
  p = (n == lp.aggpos) ? __fmul_rn(p, lp.agg) : p;
  const float q = __fmul_rn(exp2_fast(__fmaf_rn(ld, kLog2e, -k.Cd)), k.ad);
  return fmaxf(__fsub_rn(p, q), 0.f);
}

// Per-thread, per-tile partial masses, then block-wide tile totals T[k] (in sm.tile_tot).
// Mass of element j of tile t of a chunk in the tile layout: Eq. opt_G / Eq. g_tsd / p, or with LAN
// Eq. g_lantern through the thread's patch (bit t*kE + j).
template <int DT, bool XF, int kT, bool LAN>
__device__ __forceinline__ float tile_elem(const RowRegs<DT, XF, kT>& rt, const RowRegs<DT, XF, kT>& rd,
                                           const ResidCoef& k, const LanPatch& lp, int t, int j) {
  if constexpr (LAN) return resid_elem_lan(rt.get(t, j), rd.get(t, j), k, lp, t * Vec<DT>::kE + j);
  else return resid_elem(rt.get(t, j), rd.get(t, j), k);
}

template <int DT, bool XF, int kT, bool LAN = false>
__device__ __forceinline__ void chunk_masses(const RowRegs<DT, XF, kT>& rt, const RowRegs<DT, XF, kT>& rd,
                                             const ResidCoef& k, float (&part)[kT], Smem& sm,
                                             const LanPatch lp = LanPatch{0u, -1, 1.f}) {
  constexpr int kE = Vec<DT>::kE;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
  for (int t = 0; t < kT; ++t) {
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < kE; ++j) acc = __fadd_rn(acc, tile_elem<DT, XF, kT, LAN>(rt, rd, k, lp, t, j));
    part[t] = acc;
  }
  __syncthreads();  // previous readers of tile_part / tile_tot are done
#pragma unroll
  for (int t = 0; t < kT; ++t) {
    float v = wave_sum(part[t]);
    if (lane == 0) sm.tile_part[wv][t] = v;
  }
  __syncthreads();
  if (threadIdx.x < kT) {
    const int t = threadIdx.x;
    sm.tile_tot[t] = ((sm.tile_part[0][t] + sm.tile_part[1][t]) + sm.tile_part[2][t]) + sm.tile_part[3][t];
  }
  __syncthreads();
}

// Inverse CDF inside one chunk held in registers: the smallest element offset whose running
// mass (ascending token order: tile, then thread, then element) exceeds v.  Hierarchical:
// tile -> thread -> element, each level "first positive-mass entry whose inclusive sum
// exceeds the remainder, else the last positive-mass entry", so the result always has
// positive mass even when the levels' roundings disagree.  Returns the offset in the chunk
// (same value in every thread), or -1 if the chunk holds no mass.
// trust (the same in every thread): no level fell back to its last entry with mass; otherwise the
// caller re-does the draw in fp64.
template <int DT, bool XF, int kT, bool LAN = false>
__device__ __forceinline__ int chunk_select(const RowRegs<DT, XF, kT>& rt, const RowRegs<DT, XF, kT>& rd,
                                            const ResidCoef& k, const float (&part)[kT],
                                            float v, Smem& sm, bool& trust,
                                            const LanPatch lp = LanPatch{0u, -1, 1.f}) {
  constexpr int kE = Vec<DT>::kE;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  trust = false;
  // level 1: tile
  int ks = -1, klast = -1;
  float base = 0.f, base_last = 0.f, cum = 0.f;
#pragma unroll
  for (int t = 0; t < kT; ++t) {
    const float T = sm.tile_tot[t];
    if (T > 0.f) {
      if (ks < 0 && __fadd_rn(cum, T) > v) { ks = t; base = cum; }
      klast = t; base_last = cum;
    }
    cum = __fadd_rn(cum, T);
  }
  const bool tile_fallback = ks < 0;
  if (tile_fallback) { ks = klast; base = base_last; }
  if (ks < 0) return -1;
  const float v2 = v - base;
  // level 2: thread
  float my = 0.f;
#pragma unroll
  for (int t = 0; t < kT; ++t) if (t == ks) my = part[t];
  const float incl_w = wave_scan_incl(my);
  const float excl_w = wave_prev_lane(incl_w);
  if (lane == 63) sm.scan_tot[wv] = incl_w;
  __syncthreads();
  float woff = 0.f;
  for (int w = 0; w < wv; ++w) woff = __fadd_rn(woff, sm.scan_tot[w]);
  const float incl = __fadd_rn(woff, incl_w), excl = __fadd_rn(woff, excl_w);
  const bool pos = my > 0.f;
  const bool hit = pos && (incl > v2);
  const unsigned long long bh = __ballot(hit), bp = __ballot(pos);
  if (lane == 0) {
    sm.pick_first[wv] = bh ? (wv * 64 + __ffsll((long long)bh) - 1) : 0x7fffffff;
    sm.pick_last[wv] = bp ? (wv * 64 + 63 - __clzll((long long)bp)) : -1;
  }
  __syncthreads();
  int win = min(min(sm.pick_first[0], sm.pick_first[1]), min(sm.pick_first[2], sm.pick_first[3]));
  const bool thread_fallback = win == 0x7fffffff;
  if (thread_fallback) win = max(max(sm.pick_last[0], sm.pick_last[1]), max(sm.pick_last[2], sm.pick_last[3]));
  if (win < 0) return -1;
  // level 3: element, by the winning thread
  if ((int)threadIdx.x == win) {
    const float v3 = v2 - excl;
    int found = -1, last = 0;
    float run = 0.f;
#pragma unroll
    for (int t = 0; t < kT; ++t) {
      if (t == ks) {
#pragma unroll
        for (int j = 0; j < kE; ++j) {
          const float r = tile_elem<DT, XF, kT, LAN>(rt, rd, k, lp, t, j);
          if (r > 0.f) {
            last = j;
            run = __fadd_rn(run, r);
            if (found < 0 && run > v3) found = j;
          }
        }
      }
    }
    const bool element_fallback = found < 0;
    if (element_fallback) found = last;
    sm.bcast_i = (ks * kThreads + win) * kE + found;
    sm.trust = !(tile_fallback || thread_fallback || element_fallback);
  }
  __syncthreads();
  trust = sm.trust != 0;
  return sm.bcast_i;
}

// f_i = min{1, omega_i p_i(x~_i) / q_i(x~_i)} of Eq. relax from the statistics of the row pair and the
// two logits of x~_i, in fp64: the decision u_i <= f_i is made once per position, so its arithmetic
// costs nothing, and what is left of the error is that of the fp32 row sums St, Sd.  The ratio
// p/q is formed from the DIFFERENCE of the two logits (exact in fp64) and of the integer reference
// exponents, so it survives when both probabilities underflow.  A token the draft excludes (q = 0)
// has f = 1, also at 0/0; omega = 0 gives f = 0.
__device__ __forceinline__ double relaxed_accept_prob(float lt, float ld, float Ct, float St, float Cd, float Sd,
                                                      float omega) {
  if (ld == -INFINITY) return 1.0;
  if (!(omega > 0.f)) return 0.0;
  const double e = fma((double)lt - (double)ld, kLog2eD, (double)Cd - (double)Ct);
  // 2^e may exceed the fp64 range for absurd logit gaps: anything beyond 2^64 is f = 1 anyway
  const double ratio = (e > 64.0 ? 1.8446744073709552e19 : exp2_d(e)) * ((double)Sd / (double)St);
  return fmin(1.0, (double)omega * ratio);
}

// f_i of Eq. relax and the accept test of position i of sequence b, from the statistics of its row
// pair, the two logits of x~_i, omega_i and u_i.  Returns true when x~_i is rejected; a bonus row
// (has_draft false) never is.  With `emit` it writes the per-position diagnostics.
__device__ __forceinline__ bool accept_test(const KArgs& a, int b, int i, bool emit, bool has_draft, float Ct, float St,
                                            float Cd, float Sd, float lt, float ld, float omega, float u) {
  const double fi = relaxed_accept_prob(lt, ld, Ct, St, Cd, Sd, omega);
  if (emit && has_draft) {
    const int64_t o = int64_t(b) * a.L + i;
    const float et = __fmaf_rn(lt, kLog2e, -Ct), ed = __fmaf_rn(ld, kLog2e, -Cd);
    // aggregated probability of the neighbour set (Eq. p_lantern at x~_i): p_i(x~_i) times agg,
    // which the LANTERN-style call passes as omega_i
    if (a.p_agg_out) a.p_agg_out[o] = __fmul_rn(exp2_fast(et) / St, omega);
    if (a.p_tok) a.p_tok[o] = exp2_fast(et) / St;
    if (a.q_tok) a.q_tok[o] = exp2_fast(ed) / Sd;
    if (a.f) a.f[o] = (float)fi;
  }
  return has_draft && !((double)u <= fi);
}

// Position i of sequence b: statistics of its row pair (or of the bonus row alone), f_i of
// Eq. relax and the accept test.  Returns true when x~_i is rejected.  With `emit` it writes the
// per-position diagnostics.
__device__ __forceinline__ bool eval_position(const KArgs& a, int b, int i, bool emit, float& Ct, float& St,
                                              float& Cd, float& Sd) {
  // This runs in one wave while the rest of the workgroup waits for tau, so what matters is the
  // number of dependent memory round trips: everything the position needs -- the statistics of
  // both rows, the two logits of the draft token, omega_i and u_i -- is requested before the first
  // value is used, with no branch in between (the bonus row has no draft: it re-reads the last
  // draft position's entries and ignores them).
  const int rps = a.L + a.has_bonus;
  const bool has_draft = i < a.L;
  const int id = has_draft ? i : a.L - 1;
  const int rt_ = b * rps + i, rd_ = a.rows_t + b * a.L + id;
  float2 vt[kMaxDirect], vd[kMaxDirect];
  load_row_parts(a, rt_, vt);
  load_row_parts(a, rd_, vd);
  // logits of the draft token, left by the statistics kernel (nothing was left for a bonus row:
  // whatever the slot holds is read and ignored)
  const float lt = a.tok_logit[rt_], ld = a.tok_logit[rd_];
  float omega = a.omega[int64_t(b) * a.om_sb + id];
  float u = a.u_acc[int64_t(b) * a.L + id];
  // the empty statement keeps the compiler from sinking these two loads down to their uses,
  // behind the wait for the others
  asm volatile("" : "+v"(omega), "+v"(u));
  combine_parts(a, vt, Ct, St);
  combine_parts(a, vd, Cd, Sd);
  const bool rej = accept_test(a, b, i, emit, has_draft, Ct, St, Cd, Sd, lt, ld, omega, u);
  if (!has_draft) { Cd = kRefFloor; Sd = 0.f; }         // the bonus row stands alone
  return rej;
}

// Accept test at every position of sequence b (Eq. relax) and tau = first rejection (Algorithm 1)
// by the TPB threads of a workgroup.  Leaves the combined statistics (Ct, St, Cd, Sd) of the row
// that will be sampled from -- position tau+1, or the bonus row L+1 -- in *rowstat and returns tau.
// With `emit` it also writes accept_len and the per-position diagnostics.
template <int DT, bool XF, int TPB>
__device__ __forceinline__ int find_tau(const KArgs& a, int b, bool emit, int* pick /*[TPB/64]*/, float4* rowstat) {
  const int rps = a.L + a.has_bonus;
  if (__builtin_expect(rps <= 64, 1)) {
    // the usual case: one wave holds every position, the first rejection is the lowest set bit
    // of a ballot, and one barrier hands tau and the sampled row's statistics to the others
    if (threadIdx.x < 64) {
      const int i = threadIdx.x;
      float Ct = kRefFloor, St = 0.f, Cd = kRefFloor, Sd = 0.f;
      bool rej = false;
      if (i < rps) rej = eval_position(a, b, i, emit, Ct, St, Cd, Sd);
      const unsigned long long br = __ballot(rej);
      const int w = br ? __ffsll((long long)br) - 1 : a.L;
      if (i == w) *rowstat = make_float4(Ct, St, Cd, Sd);      // position w, or the bonus row when w == L
      if (i == 0) {
        pick[0] = w;
        if (emit) a.accept_len[b] = w;
      }
    }
    __syncthreads();
    return pick[0];
  }
  int first = a.L;
  for (int i0 = 0; i0 < rps; i0 += TPB) {
    const int i = i0 + threadIdx.x;
    float Ct = kRefFloor, St = 0.f, Cd = kRefFloor, Sd = 0.f;
    if (i < rps && eval_position(a, b, i, emit, Ct, St, Cd, Sd)) first = min(first, i);
    // the first rejection among positions < i0 + TPB is final once it is below that bound
    int w = wave_min_i(first);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) pick[threadIdx.x >> 6] = w;
    __syncthreads();
    w = pick[0];
#pragma unroll
    for (int q = 1; q < TPB / 64; ++q) w = min(w, pick[q]);
    const bool final = (w < i0 + TPB) || (i0 + TPB >= rps);
    if (final) {
      // the thread that owns row w (position w, or the bonus row when w == L) publishes its statistics
      if (i == w) *rowstat = make_float4(Ct, St, Cd, Sd);
      __syncthreads();
      if (emit && threadIdx.x == 0) a.accept_len[b] = w;
      return w;
    }
  }
  return a.L;   // not reached
}

// Shared memory of the kernels that run 1024 threads per sequence.
struct SmemW {
  int pick[kWavesW];
  int pick_last[kWavesW];
  float scan_tot[kWavesW];
  float4 rowstat;
  int needs64;          // the fp32 draw is not trusted: re-do it in fp64
};

}  // namespace csd
