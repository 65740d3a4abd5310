// The draw x ~ G (Algorithm 1, "Sample x ~ G*"; Eq. opt_G, Eq. g_tsd, Eq. g_lantern, or the row p
// itself) re-done in fp64 for the few sequences whose fp32 result cannot be trusted.
//
// Why.  The fast kernels form p, q and the masses [p - q f]_+ in fp32.  Their cumulative masses
// carry an absolute error of up to ~3e-7 (measured against fp64 over 6e5 draws on rows of 16384 and
// 262144 logits; it does not shrink with the law's total mass R, because it is the error of the
// probabilities that are subtracted).  In units of the uniform that is 3e-7 / R: far inside the
// 1e-6 band within which a draw may legitimately land on the neighbouring token while R is of order
// one, and outside it once p and q f nearly cancel.  Likewise R itself is good to 1e-5 relative only
// while R >= 0.03.  So a law lighter than kSafeMass = 1/16 is never drawn in fp32: the workgroup
// re-does the draw with this function -- logits widened to fp64, 2^y by a polynomial accurate to
// 1e-15, normalisers, masses and cumulative sums in fp64 -- and so it does when a level of the fp32
// search had to fall back to "the last entry with mass" (its roundings disagreed), or when the fp32
// law had no mass at all.  (Measured with the fp32 path alone: for R >= 0.1 the largest distance, in
// units of u, between the uniform and the CDF boundary at which a token differed from fp64 was
// 1.1e-7; at R = 0.03, 6e-7; at R = 0.01, 9.5e-6.)  A rejected position is reached with
// probability of about R, so such laws are rare where it matters; the common path pays one barrier
// and a flag.
//
// The routine is generic over the kernels that call it: it re-reads the row pair from memory with
// element loads (any alignment, any dtype, logit transform and top-k mask applied exactly as the
// fast path applies them, in fp32 with the same roundings), so it needs nothing the caller holds
// in registers.
#pragma once
#include "stats_kernels.h"

namespace csd {

#ifndef CSD_SAFE_MASS
#define CSD_SAFE_MASS 0.0625f
#endif
constexpr float kSafeMass = CSD_SAFE_MASS;   // laws lighter than this are always drawn in fp64
constexpr double kDustMass = 1e-14;          // fp64 laws lighter than this are rounding residue: p takes their place
// One row as the exact path reads it.
struct ExactRow {
  const char* cond;
  const char* uncond;
  float thr;            // top-k threshold (-inf: none)
  double C;             // reference exponent in base-2 units (any value near the row maximum's)
};

struct ExactJob {
  ExactRow T, D;        // target row, draft row (D.cond == nullptr: the law is p itself)
  int dt;               // kDtF32 / kDtBF16
  bool xf;              // logit transform active
  int V;
  float s, inv_T;       // guidance scale, 1/temperature
  float omega;
  int mode;             // kModeOpt / kModeVanilla / kModeP
  // Eq. g_lantern: the rejected token x~, its neighbour list and the number of members of its set
  // (nbr_row == nullptr: no patch)
  const int32_t* nbr_row;   // row lan_x of the neighbour table
  int lan_k, lan_m, lan_x;
};

template <int TPB> struct ExactSmem {
  double part[TPB / 64];
  int first[TPB / 64];
  int last[TPB / 64];
  double bcast_d;
  long long bcast_x;
};

// unnormalised weight 2^(l log2e - C) of token x of a row, from the transformed and masked fp32 logit
__device__ __forceinline__ double exact_weight(const ExactJob& J, const ExactRow& r, int64_t x) {
  const float l = token_logit_any(J.dt, r.cond, r.uncond, (int)x, J.xf, J.s, J.inv_T, r.thr);
  return exp2_d(fma((double)l, kLog2eD, -r.C));
}

// Sum of one value per thread over the workgroup, the same bits in every thread: lanes by a fixed
// butterfly whose result is taken from lane 0, waves in ascending order.
template <int TPB>
__device__ __forceinline__ double exact_block_sum(double v, ExactSmem<TPB>& sm) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  v = __shfl(v, 0, 64);
  __syncthreads();                                   // earlier readers of part are done
  if ((threadIdx.x & 63) == 0) sm.part[threadIdx.x >> 6] = v;
  __syncthreads();
  double s = 0.0;
#pragma unroll
  for (int w = 0; w < TPB / 64; ++w) s += sm.part[w];
  return s;
}

// Exclusive prefix sum over the threads in ascending order; total receives the sum of all.
template <int TPB>
__device__ __forceinline__ double exact_block_scan(double v, double& total, ExactSmem<TPB>& sm) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  double incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const double t = __shfl_up(incl, o, 64);
    if (lane >= o) incl += t;
  }
  __syncthreads();
  if (lane == 63) sm.part[wv] = incl;
  __syncthreads();
  double off = 0.0, tot = 0.0;
#pragma unroll
  for (int w = 0; w < TPB / 64; ++w) {
    off += (w < wv) ? sm.part[w] : 0.0;
    tot += sm.part[w];
  }
  total = tot;
  return off + (incl - v);
}

// Is token x a member of the rejected token's neighbour set (the first lan_m valid entries of its list)?
__device__ __forceinline__ bool exact_lan_member(const ExactJob& J, int64_t x) {
  int taken = 0;
  for (int jj = 0; jj < J.lan_k && taken < J.lan_m; ++jj) {
    const int n = J.nbr_row[jj];
    if (n < 0 || n >= J.V || n == J.lan_x) continue;
    ++taken;
    if (n == x) return true;
  }
  return false;
}

// Mass of token x under the law of the job: [p - min(q, omega p)]_+ (Eq. opt_G), [p - q]_+
// (Eq. g_tsd; with the neighbour patch of Eq. g_lantern applied to p first), or p.
__device__ __forceinline__ double exact_mass(const ExactJob& J, int mode, int64_t x, double St, double Sd, double p_agg) {
  double p = exact_weight(J, J.T, x) / St;
  if (mode == kModeP) return p;
  if (J.nbr_row != nullptr) {
    if (x == J.lan_x) p = p_agg;
    else if (exact_lan_member(J, x)) p = 0.0;
  }
  const double q = exact_weight(J, J.D, x) / Sd;
  const double qf = (mode == kModeOpt) ? fmin(q, (double)J.omega * p) : q;
  return fmax(p - qf, 0.0);
}

// One level of the search: the tokens [lo, lo + n) are split into TPB consecutive pieces, thread t
// sums piece t in ascending token order; returns the piece that holds v -- the first piece with mass
// whose inclusive cumulative mass (counted from `base`) exceeds v, else the last piece with mass, or
// -1 when no piece has any -- and leaves in `base` the mass that lies before that piece.  `total`
// receives base + the mass of the whole range.  With have_v false, v is taken as u times the total
// first (the top level, where the total is the law's mass R).
template <int TPB>
__device__ __forceinline__ int exact_level(const ExactJob& J, int mode, int64_t lo, int64_t n, double St, double Sd,
                                           double p_agg, double& base, double& total, double& v, bool have_v, float u,
                                           ExactSmem<TPB>& sm) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int64_t per = (n + TPB - 1) / TPB;
  const int64_t x0 = lo + int64_t(tid) * per, x1 = min(lo + n, x0 + per);
  double mine = 0.0;
  for (int64_t x = x0; x < x1; ++x) mine += exact_mass(J, mode, x, St, Sd, p_agg);
  double tot;
  const double excl = base + exact_block_scan<TPB>(mine, tot, sm);
  total = base + tot;
  if (!have_v) v = (double)u * total;
  const bool pos = mine > 0.0, hit = pos && (excl + mine > v);
  const unsigned long long bh = __ballot(hit), bp = __ballot(pos);
  __syncthreads();
  if (lane == 0) {
    sm.first[wv] = bh ? (wv * 64 + __ffsll((long long)bh) - 1) : 0x7fffffff;
    sm.last[wv] = bp ? (wv * 64 + 63 - __clzll((long long)bp)) : -1;
  }
  __syncthreads();
  int win = 0x7fffffff, last_pos = -1;
#pragma unroll
  for (int w = 0; w < TPB / 64; ++w) { win = min(win, sm.first[w]); last_pos = max(last_pos, sm.last[w]); }
  if (win == 0x7fffffff) win = last_pos;
  if (win < 0) return -1;
  if (tid == win) sm.bcast_d = excl;
  __syncthreads();
  base = sm.bcast_d;
  return win;
}

// The draw.  Every thread of the workgroup must call it; the token (in [0, V)) and the law's mass
// are returned in every thread.  If the law has no mass at all (no rejection is possible at this
// position: any law is optimal there) it falls back to p, as the fast path does.
template <int TPB>
__device__ __forceinline__ int exact_draw(const ExactJob& J, float u, float& R_out, ExactSmem<TPB>& sm) {
  const int tid = threadIdx.x;
  const bool has_d = J.D.cond != nullptr;
  // normalisers
  double st = 0.0, sd = 0.0;
  for (int64_t x = tid; x < J.V; x += TPB) {
    st += exact_weight(J, J.T, x);
    if (has_d) sd += exact_weight(J, J.D, x);
  }
  const double St = exact_block_sum<TPB>(st, sm);
  const double Sd = has_d ? exact_block_sum<TPB>(sd, sm) : 1.0;
  // Eq. p_lantern at the rejected token: its own probability plus its set's
  double p_agg = 0.0;
  if (J.nbr_row != nullptr && has_d) {
    double acc = 0.0;
    int taken = 0;
    for (int jj = 0; jj < J.lan_k && taken < J.lan_m; ++jj) {
      const int n = J.nbr_row[jj];
      if (n < 0 || n >= J.V || n == J.lan_x) continue;
      ++taken;
      acc += exact_weight(J, J.T, n) / St;
    }
    p_agg = exact_weight(J, J.T, J.lan_x) / St + acc;
  }
  int mode = has_d ? J.mode : kModeP;
  double base = 0.0, R = 0.0, v = 0.0;
  int win = exact_level<TPB>(J, mode, 0, J.V, St, Sd, p_agg, base, R, v, false, u, sm);
  // a mass this small is rounding residue of probabilities that coincide (fp64 probabilities near 1
  // carry ~1e-16 each): treated like no mass at all
  if (!(R > kDustMass) && mode != kModeP) {
    mode = kModeP;
    base = 0.0;
    win = exact_level<TPB>(J, mode, 0, J.V, St, Sd, p_agg, base, R, v, false, u, sm);
  }
  R_out = (float)R;
  if (win < 0) return 0;                               // a row without any finite logit: outside the contract
  int64_t per = (int64_t(J.V) + TPB - 1) / TPB;
  int64_t lo = int64_t(win) * per, n = min(per, int64_t(J.V) - lo);
  // narrow until a piece is short enough for one thread to walk
  while (n > 32) {
    double tot;
    win = exact_level<TPB>(J, mode, lo, n, St, Sd, p_agg, base, tot, v, true, u, sm);
    if (win < 0) break;                                // cannot happen: the piece was chosen for its mass
    per = (n + TPB - 1) / TPB;
    const int64_t nlo = lo + int64_t(win) * per;
    n = min(per, lo + n - nlo);
    lo = nlo;
  }
  __syncthreads();
  if (tid == 0) {
    double run = base;
    int64_t found = -1, last = lo;
    for (int64_t x = lo; x < lo + n; ++x) {
      const double m = exact_mass(J, mode, x, St, Sd, p_agg);
      if (m > 0.0) {
        last = x;
        run += m;
        if (run > v) { found = x; break; }
      }
    }
    sm.bcast_x = found >= 0 ? found : last;
  }
  __syncthreads();
  return (int)sm.bcast_x;
}

}  // namespace csd
