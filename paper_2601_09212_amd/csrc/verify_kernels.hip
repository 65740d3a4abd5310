// HIP kernels of the Cool-SD verification stage for gfx950 (MI355X).
//
// What is computed (paper notation): for every draft position i of every sequence the
// softmax statistics of the target row p_i and the draft row q_i, the relaxed acceptance
// probability f_i = min{1, omega_i p_i(x~_i)/q_i(x~_i)} (Eq. relax), the accept decision
// u_i <= f_i, the accepted length tau (Algorithm 1) and one draw from the resampling law
// G* = Norm([p - min(q, omega p)]_+) (Eq. opt_G) at the first rejected position, or from
// p_{L+1} when nothing was rejected (Algorithm 1, bonus token).
//
// Launch shapes.
//   verify_rows_kernel      grid = rows x nchunks, rows = B*(L+has_bonus).  One workgroup
//                           owns one chunk (<= 16384 logits) of one (target, draft) row pair
//                           and keeps it in registers, so HBM is read exactly once.
//     nchunks == 1 : fully fused.  The workgroup finishes the row: accept test, and -- only
//                    if the row is rejected (or is the bonus row) -- the residual mass and
//                    the inverse-CDF draw from registers.  The last workgroup of a sequence
//                    to finish (completion counter) does the first-rejection scan and
//                    writes tau and x_{tau+1}.  One launch per verify call.
//     nchunks  > 1 : the workgroup publishes its partial (reference exponent, sum); the last
//                    chunk of a row combines them and does the accept test; the last row of
//                    a sequence writes tau.  resample_chunks_kernel then re-reads only the
//                    one row pair per sequence that is sampled from.
//   resample_chunks_kernel  grid = B x nchunks.
//
// No workgroup ever waits for another one: cross-workgroup hand-over uses "last one to
// arrive does the work" counters, which the last arriver resets to zero.
//
// Hand-over protocol.  Device-wide release/acquire fences write back and invalidate the whole
// L2 of an XCD and cost far more than this kernel's memory traffic, so none is used.  Instead
// every value that another workgroup of the same launch will read is written with an
// agent-scope atomic store and read with an agent-scope atomic load (both bypass the
// per-XCD L2), by one thread, which waits for its stores to complete (s_waitcnt vmcnt(0))
// before it takes its ticket with an agent-scope atomic add.  The reader only reads after
// it has seen the final ticket value.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "device_utils.h"
#include "kernels.h"

namespace csd {

enum { kModeOpt = 0, kModeVanilla = 1, kModeP = 2 };

struct Smem {
  float red_c[2][kWaves];
  float red_s[2][kWaves];
  float tile_part[kWaves][16];
  float tile_tot[16];
  float scan_tot[kWaves];
  int pick_first[kWaves];
  int pick_last[kWaves];
  int bcast_i;
  int flag;
};

template <typename T> __device__ __forceinline__ T coherent_load(const T* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ __forceinline__ void coherent_store(T* p, T v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Called by ONE thread after its coherent stores: waits until they have completed, then takes
// a ticket.  Returns true for the last of n arrivals.
__device__ __forceinline__ bool ticket_is_last(uint32_t* counter, uint32_t n) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  const uint32_t old = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  asm volatile("" ::: "memory");
  return old == n - 1u;
}

// Wave-0-only tail of a row: publish the accept decision, take the sequence's ticket and, as
// the last row of the sequence, find tau = first rejected position (Algorithm 1's break) and
// emit the outputs.  Must be called by all 64 lanes of wave 0.
__device__ __forceinline__ void finish_sequence(const KArgs& a, int b, int i, bool bonus, int acc,
                                                bool have_cand, int cand, float R, bool fused) {
  const int lane = threadIdx.x;
  const int rps = a.L + a.has_bonus;
  int last = 0;
  if (lane == 0) {
    if (!bonus) coherent_store(&a.acc[int64_t(b) * a.L + i], acc);
    if (have_cand) {
      coherent_store(&a.cand_tok[int64_t(b) * (a.L + 1) + i], cand);
      coherent_store(&a.cand_R[int64_t(b) * (a.L + 1) + i], R);
    }
    last = ticket_is_last(&a.seq_counter[b], (uint32_t)rps) ? 1 : 0;
  }
  last = __shfl(last, 0, 64);
  if (!last) return;
  int first = a.L;
  for (int j = lane; j < a.L; j += 64)
    if (coherent_load(&a.acc[int64_t(b) * a.L + j]) == 0) first = min(first, j);
  const int tau = wave_min_i(first);
  if (lane == 0) {
    a.accept_len[b] = tau;
    coherent_store(&a.seq_counter[b], 0u);
    coherent_store(&a.hint[b], 0u);
    if (fused) {
      int tok = -1;
      float mass = 0.f;
      if (tau < a.L || a.has_bonus) {
        tok = coherent_load(&a.cand_tok[int64_t(b) * (a.L + 1) + tau]);
        mass = coherent_load(&a.cand_R[int64_t(b) * (a.L + 1) + tau]);
      }
      a.next_token[b] = tok;
      if (a.resid_mass) a.resid_mass[b] = mass;
    }
  }
}

// Block-wide combine of per-thread (c, s) pairs of two rows.  Result in every thread.
__device__ __forceinline__ void block_stats(float c0, float s0, float c1, float s1, Smem& sm,
                                            float& C0, float& S0, float& C1, float& S1) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  float w0 = wave_max(c0), w1 = wave_max(c1);
  if (lane == 0) { sm.red_c[0][wv] = w0; sm.red_c[1][wv] = w1; }
  __syncthreads();
  C0 = fmaxf(fmaxf(sm.red_c[0][0], sm.red_c[0][1]), fmaxf(sm.red_c[0][2], sm.red_c[0][3]));
  C1 = fmaxf(fmaxf(sm.red_c[1][0], sm.red_c[1][1]), fmaxf(sm.red_c[1][2], sm.red_c[1][3]));
  float t0 = wave_sum(s0 * exp2_fast(c0 - C0));   // exact power-of-two rescale
  float t1 = wave_sum(s1 * exp2_fast(c1 - C1));
  if (lane == 0) { sm.red_s[0][wv] = t0; sm.red_s[1][wv] = t1; }
  __syncthreads();
  S0 = ((sm.red_s[0][0] + sm.red_s[0][1]) + sm.red_s[0][2]) + sm.red_s[0][3];
  S1 = ((sm.red_s[1][0] + sm.red_s[1][1]) + sm.red_s[1][2]) + sm.red_s[1][3];
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

// Per-thread, per-tile partial masses, then block-wide tile totals T[k] (in sm.tile_tot).
template <int DT, bool XF>
__device__ __forceinline__ void chunk_masses(const RowRegs<DT, XF>& rt, const RowRegs<DT, XF>& rd,
                                             const ResidCoef& k, float (&part)[Vec<DT>::kT], Smem& sm) {
  constexpr int kE = Vec<DT>::kE, kT = Vec<DT>::kT;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
  for (int t = 0; t < kT; ++t) {
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < kE; ++j) acc = __fadd_rn(acc, resid_elem(rt.get(t, j), rd.get(t, j), k));
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

// Sum of the tile totals in ascending order (the chunk's mass).
template <int kT> __device__ __forceinline__ float chunk_total(const Smem& sm) {
  float R = 0.f;
#pragma unroll
  for (int t = 0; t < kT; ++t) R = __fadd_rn(R, sm.tile_tot[t]);
  return R;
}

// Inverse CDF inside one chunk held in registers: the smallest element offset whose running
// mass (ascending token order: tile, then thread, then element) exceeds v.  Hierarchical:
// tile -> thread -> element, each level "first positive-mass entry whose inclusive sum
// exceeds the remainder, else the last positive-mass entry", so the result always has
// positive mass even when the levels' roundings disagree.  Returns the offset in the chunk
// (same value in every thread), or -1 if the chunk holds no mass.
template <int DT, bool XF>
__device__ __forceinline__ int chunk_select(const RowRegs<DT, XF>& rt, const RowRegs<DT, XF>& rd,
                                            const ResidCoef& k, const float (&part)[Vec<DT>::kT],
                                            float v, Smem& sm) {
  constexpr int kE = Vec<DT>::kE, kT = Vec<DT>::kT;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
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
  if (ks < 0) { ks = klast; base = base_last; }
  if (ks < 0) return -1;
  const float v2 = v - base;
  // level 2: thread
  float my = 0.f;
#pragma unroll
  for (int t = 0; t < kT; ++t) if (t == ks) my = part[t];
  const float incl_w = wave_scan_incl(my);
  float excl_w = __shfl_up(incl_w, 1, 64);
  if (lane == 0) excl_w = 0.f;
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
  if (win == 0x7fffffff) win = max(max(sm.pick_last[0], sm.pick_last[1]), max(sm.pick_last[2], sm.pick_last[3]));
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
          const float r = resid_elem(rt.get(t, j), rd.get(t, j), k);
          if (r > 0.f) {
            last = j;
            run = __fadd_rn(run, r);
            if (found < 0 && run > v3) found = j;
          }
        }
      }
    }
    if (found < 0) found = last;
    sm.bcast_i = (ks * kThreads + win) * kE + found;
  }
  __syncthreads();
  return sm.bcast_i;
}

__device__ __forceinline__ const char* row_ptr(const void* base, int64_t elem_off, int es) {
  return base ? reinterpret_cast<const char*>(base) + elem_off * es : nullptr;
}

// Transformed logit of one token of a row (scalar path, used for x~_i).
template <int DT>
__device__ __forceinline__ float token_logit(const char* cond, const char* uncond, int x, bool xf,
                                             float s, float inv_T) {
  float lc = load_elem<DT>(cond, x);
  if (!xf) return lc;
  float lu = uncond ? load_elem<DT>(uncond, x) : 0.f;
  return transform_logit(lc, lu, uncond != nullptr, s, inv_T);
}

template <int DT, bool XF, bool AL>
__global__ __launch_bounds__(kThreads) void verify_rows_kernel(const KArgs a) {
  constexpr int kT = Vec<DT>::kT, kES = Vec<DT>::kES;
  __shared__ Smem sm;
  const int C = a.nchunks;
  const int row = blockIdx.x / C, c = blockIdx.x - row * C;
  const int rps = a.L + a.has_bonus;
  const int b = row / rps, i = row - b * rps;
  const bool bonus = a.resample_only ? (a.d == nullptr) : (i == a.L);
  const int64_t base = int64_t(c) * kChunk;

  const char* t_c = row_ptr(a.t, int64_t(b) * a.t_sb + int64_t(i) * a.t_sl, kES);
  const char* t_u = row_ptr(a.tu, int64_t(b) * a.t_sb + int64_t(i) * a.t_sl, kES);
  const char* d_c = bonus ? nullptr : row_ptr(a.d, int64_t(b) * a.d_sb + int64_t(i) * a.d_sl, kES);
  const char* d_u = bonus ? nullptr : row_ptr(a.du, int64_t(b) * a.d_sb + int64_t(i) * a.d_sl, kES);

  RowRegs<DT, XF> rt, rd;
  load_chunk<DT, XF, AL>(rt, t_c, t_u, base, a.V, a.cfg_scale, a.inv_T);
  if (!bonus) {
    load_chunk<DT, XF, AL>(rd, d_c, d_u, base, a.V, a.cfg_scale, a.inv_T);
  } else {
#pragma unroll
    for (int n = 0; n < RowRegs<DT, XF>::kWords; ++n) rd.w[n] = 0u;   // never read in mode P
  }

  float ct, st, cd = kRefFloor, sd = 0.f;
  thread_stats<DT, XF>(rt, ct, st);
  if (!bonus) thread_stats<DT, XF>(rd, cd, sd);
  float Ct, St, Cd, Sd;
  block_stats(ct, st, cd, sd, sm, Ct, St, Cd, Sd);

  if (C > 1) {
    // publish the chunk's partial statistics; the last chunk of the row combines them
    if (threadIdx.x >= 64) return;                 // the rest is scalar work for wave 0
    int last = 0;
    if (threadIdx.x == 0) {
      float4* pp = &a.part[int64_t(row) * C + c];
      coherent_store(&pp->x, Ct); coherent_store(&pp->y, St);
      coherent_store(&pp->z, Cd); coherent_store(&pp->w, Sd);
      last = ticket_is_last(&a.row_counter[row], (uint32_t)C) ? 1 : 0;
    }
    if (!__shfl(last, 0, 64)) return;
    float mt = kRefFloor, md = kRefFloor;
    for (int cc = 0; cc < C; ++cc) {
      mt = fmaxf(mt, coherent_load(&a.part[int64_t(row) * C + cc].x));
      md = fmaxf(md, coherent_load(&a.part[int64_t(row) * C + cc].z));
    }
    float sst = 0.f, ssd = 0.f;
    for (int cc = 0; cc < C; ++cc) {
      const float4* pp = &a.part[int64_t(row) * C + cc];
      sst = __fadd_rn(sst, coherent_load(&pp->y) * exp2_fast(coherent_load(&pp->x) - mt));
      ssd = __fadd_rn(ssd, coherent_load(&pp->w) * exp2_fast(coherent_load(&pp->z) - md));
    }
    Ct = mt; St = sst; Cd = md; Sd = ssd;
    if (threadIdx.x == 0) {
      coherent_store(&a.row_counter[row], 0u);
      a.rowstat[row] = make_float4(Ct, St, Cd, Sd);   // read by the next kernel only
    }
  }

  // ---- row level: acceptance test of position i (Eq. relax, Algorithm 1)
  int acc = 1;
  const float omega = bonus ? 1.f : a.omega[int64_t(b) * a.om_sb + i];
  if (!bonus && !a.resample_only) {
    int x = a.tokens[int64_t(b) * a.L + i];
    x = min(max(x, 0), a.V - 1);
    float lt = token_logit<DT>(t_c, t_u, x, XF, a.cfg_scale, a.inv_T);
    float ld = token_logit<DT>(d_c, d_u, x, XF, a.cfg_scale, a.inv_T);
    // exponents of p(x~) and q(x~) in base-2 units; the ratio p/q is formed from their
    // difference so that it survives when both probabilities underflow fp32
    const float et = __fmaf_rn(lt, kLog2e, -Ct), ed = __fmaf_rn(ld, kLog2e, -Cd);
    const float p_x = exp2_fast(et) / St;
    const float q_x = exp2_fast(ed) / Sd;
    const float ratio = __fmul_rn(exp2_fast(__fsub_rn(et, ed)), Sd / St);
    // f = min{1, omega p/q}; a token the draft excludes (q = 0) has f = 1, also at 0/0
    const float fi = (ld == -INFINITY) ? 1.f : ((omega > 0.f) ? fminf(1.f, __fmul_rn(omega, ratio)) : 0.f);
    const float u = a.u_acc[int64_t(b) * a.L + i];
    acc = (u <= fi) ? 1 : 0;
    if (threadIdx.x == 0) {
      const int64_t o = int64_t(b) * a.L + i;
      if (a.p_tok) a.p_tok[o] = p_x;
      if (a.q_tok) a.q_tok[o] = q_x;
      if (a.f) a.f[o] = fi;
    }
  } else if (a.resample_only) {
    acc = 0;
  }

  if (C > 1) {                                     // wave 0 of the row's last chunk
    if (!a.resample_only) finish_sequence(a, b, i, bonus, acc, false, -1, 0.f, false);
    return;
  }

  // ---- does this row's resampling law have to be sampled?  Only the FIRST rejected position
  // of a sequence is (Algorithm 1 breaks there), or the bonus row if nothing is rejected.  A
  // rejected row raises hint[b] to L - i and skips the work if an earlier position already
  // raised it higher; the bonus row skips if any position did.  The first rejected position
  // never skips, whatever the order in which workgroups run.
  bool need = a.resample_only != 0;
  if (!need && (bonus || acc == 0)) {
    if (threadIdx.x == 0) {
      uint32_t mine = bonus ? 0u : uint32_t(a.L - i);
      uint32_t old = bonus ? coherent_load(&a.hint[b])
                           : __hip_atomic_fetch_max(&a.hint[b], mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      sm.flag = bonus ? (old == 0u) : (mine > old);
    }
    __syncthreads();
    need = sm.flag != 0;
  }

  // ---- candidate draw from this row's resampling law (Eq. opt_G / Eq. g_tsd / p_{L+1})
  int cand = -1;
  float R = 0.f;
  if (need) {
    ResidCoef k{Ct, 1.f / St, Cd, bonus ? 1.f : 1.f / Sd, omega,
                bonus ? kModeP : (a.resample_mode == 1 ? kModeVanilla : kModeOpt)};
    float part[kT];
    chunk_masses<DT, XF>(rt, rd, k, part, sm);
    R = chunk_total<kT>(sm);
    if (!(R > 0.f)) {  // no rejection possible at this position: any law is optimal, use p
      k.mode = kModeP;
      chunk_masses<DT, XF>(rt, rd, k, part, sm);
      R = chunk_total<kT>(sm);
    }
    const float u = a.u_res[b];
    cand = chunk_select<DT, XF>(rt, rd, k, part, __fmul_rn(u, R), sm);
    if (cand >= a.V) cand = a.V - 1;
  }

  if (a.resample_only) {
    if (threadIdx.x == 0) {
      a.next_token[b] = cand;
      if (a.resid_mass) a.resid_mass[b] = R;
    }
    return;
  }
  if (threadIdx.x >= 64) return;
  finish_sequence(a, b, i, bonus, acc, need, cand, R, true);
}

// Second kernel of the chunked path: per sequence, draw x_{tau+1} from the resampling law of
// row tau+1 (Eq. opt_G), whose logits are re-read once.  Workgroup (b, c) computes the mass of
// chunk c; the last one to finish picks the chunk that contains u*R and searches it.
template <int DT, bool XF, bool AL>
__global__ __launch_bounds__(kThreads) void resample_chunks_kernel(const KArgs a) {
  constexpr int kT = Vec<DT>::kT, kES = Vec<DT>::kES;
  __shared__ Smem sm;
  const int C = a.nchunks;
  const int b = blockIdx.x / C, c = blockIdx.x - b * C;
  const int rps = a.L + a.has_bonus;
  const int j = a.resample_only ? 0 : a.accept_len[b];
  if (!a.resample_only && j >= a.L && !a.has_bonus) {
    if (c == 0 && threadIdx.x == 0) {
      a.next_token[b] = -1;
      if (a.resid_mass) a.resid_mass[b] = 0.f;
    }
    return;
  }
  const bool bonus = a.resample_only ? (a.d == nullptr) : (j == a.L);
  const int row = b * rps + j;
  const char* t_c = row_ptr(a.t, int64_t(b) * a.t_sb + int64_t(j) * a.t_sl, kES);
  const char* t_u = row_ptr(a.tu, int64_t(b) * a.t_sb + int64_t(j) * a.t_sl, kES);
  const char* d_c = bonus ? nullptr : row_ptr(a.d, int64_t(b) * a.d_sb + int64_t(j) * a.d_sl, kES);
  const char* d_u = bonus ? nullptr : row_ptr(a.du, int64_t(b) * a.d_sb + int64_t(j) * a.d_sl, kES);
  const float4 rs = a.rowstat[row];
  const float omega = bonus ? 1.f : a.omega[int64_t(b) * a.om_sb + j];
  ResidCoef k{rs.x, 1.f / rs.y, rs.z, bonus ? 1.f : 1.f / rs.w, omega,
              bonus ? kModeP : (a.resample_mode == 1 ? kModeVanilla : kModeOpt)};

  RowRegs<DT, XF> rt, rd;
  float part[kT];
  auto load_pair = [&](int cc) {
    const int64_t base = int64_t(cc) * kChunk;
    load_chunk<DT, XF, AL>(rt, t_c, t_u, base, a.V, a.cfg_scale, a.inv_T);
    if (!bonus) {
      load_chunk<DT, XF, AL>(rd, d_c, d_u, base, a.V, a.cfg_scale, a.inv_T);
    } else {
#pragma unroll
      for (int n = 0; n < RowRegs<DT, XF>::kWords; ++n) rd.w[n] = 0u;
    }
  };
  load_pair(c);
  chunk_masses<DT, XF>(rt, rd, k, part, sm);
  const float Rc = chunk_total<kT>(sm);
  if (threadIdx.x == 0) {
    coherent_store(&a.chunk_R[int64_t(b) * C + c], Rc);
    sm.flag = ticket_is_last(&a.k2_counter[b], (uint32_t)C) ? 1 : 0;
  }
  __syncthreads();
  if (!sm.flag) return;

  // total mass over the chunks, ascending
  float R = 0.f;
  for (int cc = 0; cc < C; ++cc) R = __fadd_rn(R, coherent_load(&a.chunk_R[int64_t(b) * C + cc]));
  const bool fallback = !(R > 0.f);   // no rejection possible here: any law is optimal, use p
  auto chunk_mass = [&](int cc) -> float {
    if (!fallback) return coherent_load(&a.chunk_R[int64_t(b) * C + cc]);
    const float4 pp = a.part[int64_t(row) * C + cc];
    return __fmul_rn(__fmul_rn(pp.y, exp2_fast(pp.x - rs.x)), k.at);
  };
  if (fallback) {
    k.mode = kModeP;
    R = 0.f;
    for (int cc = 0; cc < C; ++cc) R = __fadd_rn(R, chunk_mass(cc));
  }
  const float v = __fmul_rn(a.u_res[b], R);
  int cs = -1, clast = -1;
  float cbase = 0.f, cbase_last = 0.f, cum = 0.f;
  for (int cc = 0; cc < C; ++cc) {
    const float m = chunk_mass(cc);
    if (m > 0.f) {
      if (cs < 0 && __fadd_rn(cum, m) > v) { cs = cc; cbase = cum; }
      clast = cc; cbase_last = cum;
    }
    cum = __fadd_rn(cum, m);
  }
  if (cs < 0) { cs = clast; cbase = cbase_last; }
  int token = 0;
  if (cs >= 0) {
    if (cs != c || fallback) {
      __syncthreads();
      load_pair(cs);
      chunk_masses<DT, XF>(rt, rd, k, part, sm);
    }
    const int off = chunk_select<DT, XF>(rt, rd, k, part, v - cbase, sm);
    token = cs * kChunk + max(off, 0);
  }
  if (token >= a.V) token = a.V - 1;
  if (threadIdx.x == 0) {
    a.next_token[b] = token;
    if (a.resid_mass) a.resid_mass[b] = R;
    coherent_store(&a.k2_counter[b], 0u);
  }
}

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

template <int DT, bool XF, bool AL>
static hipError_t launch_typed(const KArgs& a, hipStream_t stream) {
  (void)hipGetLastError();
  const int64_t rows = a.resample_only ? int64_t(a.B) : int64_t(a.B) * (a.L + a.has_bonus);
  const int64_t grid1 = rows * a.nchunks;
  hipLaunchKernelGGL((verify_rows_kernel<DT, XF, AL>), dim3((unsigned)grid1), dim3(kThreads), 0, stream, a);
  hipError_t e = checked("verify_rows_kernel");
  if (e != hipSuccess) return e;
  if (a.nchunks > 1) {
    const int64_t grid2 = int64_t(a.B) * a.nchunks;
    hipLaunchKernelGGL((resample_chunks_kernel<DT, XF, AL>), dim3((unsigned)grid2), dim3(kThreads), 0, stream, a);
    e = checked("resample_chunks_kernel");
  }
  return e;
}

template <int DT, bool XF>
static hipError_t launch_al(const KArgs& a, hipStream_t stream) {
  return a.aligned ? launch_typed<DT, XF, true>(a, stream) : launch_typed<DT, XF, false>(a, stream);
}

hipError_t launch_verify(const KArgs& a, int dtype, bool xf, hipStream_t stream) {
  if (dtype == kDtBF16) return xf ? launch_al<kDtBF16, true>(a, stream) : launch_al<kDtBF16, false>(a, stream);
  return xf ? launch_al<kDtF32, true>(a, stream) : launch_al<kDtF32, false>(a, stream);
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
