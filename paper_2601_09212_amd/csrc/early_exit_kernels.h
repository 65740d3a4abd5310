// Early-exit form of the verify call and the one-launch cool_sd_resample on short rows.
#pragma once
#include "sequence_whole.h"

namespace csd {

// ============================================================================ early-exit variant
// Algorithm 1 stops verifying at the first rejection; this kernel does the same with the memory
// traffic: one workgroup of 1024 threads per sequence walks the positions in order, holds the
// current (target, draft) row pair in registers, forms its softmax statistics and the accept
// test, and on the first rejection draws x_{tau+1} from the pair it already holds.  Rows after
// the rejected position are never read, except the one pair whose loads were issued ahead while
// the current pair was being processed.  For 16-byte aligned rows of at most 16384 logits,
// L <= kMaxLEarly and no top-k.  Per-position outputs after the rejected position are set to NaN.
constexpr int kMaxLEarly = 1024;

struct RedW {
  float red_c[2][2][kWavesW];    // [step parity][target / draft][wave]
  float red_s[2][2][kWavesW];
};
struct SmemE {
  SmemW w;
  RedW red;
  float tokl[2][2];              // [step parity][target / draft] logit of the draft token
  int tok[kMaxLEarly];
  float u[kMaxLEarly];
  float om[kMaxLEarly];
};

// Block-wide softmax statistics of a row spread over 1024 threads: per-thread (c, s) are reduced
// per wave and left in LDS (slot par, row which); after the caller's barrier block_stats_read
// combines the 16 wave entries (reference = max, sums rescaled by exact powers of two, fixed tree).
template <int DT, bool XF, int kVW>
__device__ __forceinline__ void block_stats_write(const RowRegs<DT, XF, kVW>& r, RedW& sm, int par, int which) {
  float c, s;
  thread_stats<DT, XF, kVW>(r, c, s);
  const float wc = wave_max(c);
  const float ws = wave_sum(s * exp2_fast(c - wc));
  if ((threadIdx.x & 63) == 0) { sm.red_c[par][which][threadIdx.x >> 6] = wc; sm.red_s[par][which][threadIdx.x >> 6] = ws; }
}
__device__ __forceinline__ void block_stats_read(const RedW& sm, int par, int which, float& C, float& S) {
  // every wave reduces the 16 entries for itself, one per lane, instead of every thread reading all
  const int lane = threadIdx.x & 63;
  const float c = lane < kWavesW ? sm.red_c[par][which][lane] : kRefFloor;
  const float s = lane < kWavesW ? sm.red_s[par][which][lane] : 0.f;
  C = wave_max(c);
  S = wave_sum(s * exp2_fast(c - C));
}

// D: row pairs in flight ahead of the one being processed (a ring of register slots; the loop is
// unrolled by D so that every slot is a fixed set of registers).  One is what is used: a step is
// bound by its arithmetic and its barrier (about 3 us for 16 waves sharing one compute unit), not
// by the load latency, so deeper rings only cost registers and read more unneeded pairs.
template <int DT, bool XF, int D>
__global__ __launch_bounds__(kThreadsW) void sequence_early_exit_kernel(const KArgs a) {
  constexpr int kE = Vec<DT>::kE, kES = Vec<DT>::kES;
  constexpr int kVW = kChunk / (kThreadsW * kE);       // vectors per thread: 2 (bf16) / 4 (fp32)
  constexpr int kPer = kVW * kE;                       // logits per thread
  __shared__ SmemE sm;
  __shared__ ExactSmem<kThreadsW> smx;
  const int b = blockIdx.x, L = a.L, tid = threadIdx.x;
  if (tid == 0) sm.w.needs64 = 0;
  for (int i = tid; i < L; i += kThreadsW) {
    sm.tok[i] = min(max(a.tokens[int64_t(b) * L + i], 0), a.V - 1);
    sm.u[i] = a.u_acc[int64_t(b) * L + i];
    sm.om[i] = a.omega[int64_t(b) * a.om_sb + i];
  }
  // pair i < L: target and draft row of position i+1; "pair" L: the bonus row alone.  A slot
  // holds the fetched vectors untouched, so nothing waits for them until the pair's turn comes.
  struct Slot { uint4 tc[kVW], dc[kVW], tu[kVW], du[kVW]; };   // tu / du stay unused without a logit transform
  const bool guided = XF && a.tu != nullptr;
  int64_t first[kVW];
#pragma unroll
  for (int v = 0; v < kVW; ++v) first[v] = int64_t(tid * kVW + v) * kE;
  // Always the same number of loads, whatever i is (row indices are clamped to the last valid row,
  // whose re-read is harmless): the compiler can then count how many younger loads are in flight
  // and wait only for the slot being consumed.
  auto fetch_pair = [&](Slot& sl, int i) {
    const int it = min(i, L + a.has_bonus - 1), id = min(i, L - 1);
    const int64_t ot = int64_t(b) * a.t_sb + int64_t(it) * a.t_sl;
    const int64_t od = int64_t(b) * a.d_sb + int64_t(id) * a.d_sl;
    const char* tc = row_ptr(a.t, ot, kES);
    const char* dc = row_ptr(a.d, od, kES);
    const char* tu = guided ? row_ptr(a.tu, ot, kES) : tc;
    const char* du = guided ? row_ptr(a.du, od, kES) : dc;
#pragma unroll
    for (int v = 0; v < kVW; ++v) {
      sl.tc[v] = fetch_vec<DT>(tc, first[v], a.V);
      sl.dc[v] = fetch_vec<DT>(dc, first[v], a.V);
      if constexpr (XF) {
        sl.tu[v] = fetch_vec<DT>(tu, first[v], a.V);
        sl.du[v] = fetch_vec<DT>(du, first[v], a.V);
      }
    }
  };
  Slot slot[D];
#pragma unroll
  for (int s = 0; s < D; ++s) {
#pragma unroll
    for (int v = 0; v < kVW; ++v) {
      slot[s].tc[v] = slot[s].dc[v] = slot[s].tu[v] = slot[s].du[v] = make_uint4(0u, 0u, 0u, 0u);
    }
    fetch_pair(slot[s], s);
  }
  RowRegs<DT, XF, kVW> rt, rd;
  rt.clear();
  rd.clear();
  __syncthreads();                                      // tok / u / om are visible

  int j = L;                                            // first rejected position
  float Ct = kRefFloor, St = 1.f, Cd = kRefFloor, Sd = 1.f;
  // One verification step on the pair in slot sl (position i); true = rejected.
  auto step = [&](Slot& sl, int i) -> bool {
    finish_chunk<DT, XF, kVW>(rt, sl.tc, sl.tu, first, a.V, guided, a.cfg_scale, a.inv_T, -INFINITY);
    finish_chunk<DT, XF, kVW>(rd, sl.dc, sl.du, first, a.V, guided, a.cfg_scale, a.inv_T, -INFINITY);
    fetch_pair(sl, i + D);                              // refill the slot before working on the pair
    const int par = i & 1;
    block_stats_write<DT, XF, kVW>(rt, sm.red, par, 0);
    block_stats_write<DT, XF, kVW>(rd, sm.red, par, 1);
    // the thread that holds x~_i publishes its two logits
    const int idx = sm.tok[i] - tid * kPer;
    float lt = 0.f, ld = 0.f;
    if ((sm.tok[i] >> 6) / kPer == (tid >> 6)) {        // only the wave that holds the token looks for it
#pragma unroll
      for (int v = 0; v < kVW; ++v) {
#pragma unroll
        for (int e = 0; e < kE; ++e) {
          if (idx == v * kE + e) { lt = rt.get(v, e); ld = rd.get(v, e); }
        }
      }
      if (idx >= 0 && idx < kPer) { sm.tokl[par][0] = lt; sm.tokl[par][1] = ld; }
    }
    __syncthreads();       // the only barrier of a step: LDS slots alternate with the step parity
    block_stats_read(sm.red, par, 0, Ct, St);
    block_stats_read(sm.red, par, 1, Cd, Sd);
    lt = sm.tokl[par][0];
    ld = sm.tokl[par][1];
    // same evaluation of f_i = min{1, omega_i p_i(x~_i) / q_i(x~_i)} as the all-rows path (Eq. relax)
    const double fi = relaxed_accept_prob(lt, ld, Ct, St, Cd, Sd, sm.om[i]);
    if (tid == 0) {
      const int64_t o = int64_t(b) * L + i;
      const float et = __fmaf_rn(lt, kLog2e, -Ct), ed = __fmaf_rn(ld, kLog2e, -Cd);
      if (a.p_tok) a.p_tok[o] = exp2_fast(et) / St;
      if (a.q_tok) a.q_tok[o] = exp2_fast(ed) / Sd;
      if (a.f) a.f[o] = (float)fi;
    }
    return !((double)sm.u[i] <= fi);                            // uniform: every thread sees the same values
  };
  for (int i0 = 0; i0 < L && j == L; i0 += D) {
#pragma unroll
    for (int s = 0; s < D; ++s) {
      if (j == L && i0 + s < L) {
        if (step(slot[s], i0 + s)) j = i0 + s;
      }
    }
  }
  // positions that were never evaluated
  for (int i = j + 1 + tid; i < L; i += kThreadsW) {
    const int64_t o = int64_t(b) * L + i;
    if (a.p_tok) a.p_tok[o] = NAN;
    if (a.q_tok) a.q_tok[o] = NAN;
    if (a.f) a.f[o] = NAN;
  }
  if (tid == 0) a.accept_len[b] = j;
  const bool bonus = j == L;
  if (bonus) {
    if (!a.has_bonus) {
      if (tid == 0) {
        a.next_token[b] = -1;
        if (a.resid_mass) a.resid_mass[b] = 0.f;
      }
      return;
    }
    // everything was accepted: fetch row L+1 now (its statistics go to the LDS slot of parity
    // L & 1, last used two steps ago or never)
    fetch_pair(slot[0], L);
    finish_chunk<DT, XF, kVW>(rt, slot[0].tc, slot[0].tu, first, a.V, guided, a.cfg_scale, a.inv_T, -INFINITY);
    block_stats_write<DT, XF, kVW>(rt, sm.red, L & 1, 0);
    __syncthreads();
    block_stats_read(sm.red, L & 1, 0, Ct, St);
  }
  ResidCoef k{Ct, 1.f / St, Cd, bonus ? 1.f : 1.f / Sd, bonus ? 1.f : sm.om[j],
              bonus ? kModeP : (a.resample_mode == 1 ? kModeVanilla : kModeOpt)};
  float R;
  bool writer, trust;
  int token = sample_whole<DT, XF, kVW>(rt, rd, k, a.u_res[b], a.V, sm.w, R, writer, trust);
  if (draw_needs_fp64(writer, trust, a.exact_draw, &sm.w.needs64)) {
    const int jt = bonus ? L : j;                       // the row that was sampled from
    const int64_t ot = int64_t(b) * a.t_sb + int64_t(jt) * a.t_sl, od = int64_t(b) * a.d_sb + int64_t(min(jt, L - 1)) * a.d_sl;
    const ExactJob job{{row_ptr(a.t, ot, kES), guided ? row_ptr(a.tu, ot, kES) : nullptr, -INFINITY, (double)Ct},
                       {bonus ? nullptr : row_ptr(a.d, od, kES), (guided && !bonus) ? row_ptr(a.du, od, kES) : nullptr,
                        -INFINITY, (double)Cd},
                       DT, XF, a.V, a.cfg_scale, a.inv_T, k.omega, k.mode, nullptr, 0, 0, 0};
    token = exact_draw<kThreadsW>(job, a.u_res[b], R, smx);
    writer = tid == 0;
  }
  if (writer) {
    a.next_token[b] = token;
    if (a.resid_mass) a.resid_mass[b] = R;
  }
}

// cool_sd_resample on rows of at most 16384 logits without top-k, in ONE launch: a workgroup of
// 1024 threads holds the row pair (or the single row when no draft is given), forms its softmax
// statistics block-wide and draws the token from the registers.  The drafting loop calls this once
// per drafted token, so its latency (one launch instead of two) is what matters.
// MUL = 2: rows of up to 32768 logits (32 words per row and thread), as in sequence_whole_kernel.
template <int DT, bool XF, bool AL, int MUL = 1>
__global__ __launch_bounds__(kThreadsW) void resample_whole_kernel(const KArgs a) {
  constexpr int kE = Vec<DT>::kE, kES = Vec<DT>::kES;
  constexpr int kVW = MUL * kChunk / (kThreadsW * kE);
  __shared__ SmemW sm;
  __shared__ RedW red;
  __shared__ ExactSmem<kThreadsW> smx;
  const int b = blockIdx.x;
  if (threadIdx.x == 0) sm.needs64 = 0;
  const bool bonus = a.d == nullptr;                    // no draft: the law is p itself
  const char* t_c = row_ptr(a.t, int64_t(b) * a.t_sb, kES);
  const char* t_u = row_ptr(a.tu, int64_t(b) * a.t_sb, kES);
  const char* d_c = bonus ? nullptr : row_ptr(a.d, int64_t(b) * a.d_sb, kES);
  const char* d_u = bonus ? nullptr : row_ptr(a.du, int64_t(b) * a.d_sb, kES);
  RowRegs<DT, XF, kVW> rt, rd;
  load_chunk<DT, XF, AL, kVW, 1, kVW>(rt, t_c, t_u, 0, a.V, a.cfg_scale, a.inv_T, -INFINITY);
  if (!bonus) load_chunk<DT, XF, AL, kVW, 1, kVW>(rd, d_c, d_u, 0, a.V, a.cfg_scale, a.inv_T, -INFINITY);
  else rd.clear();
  const float omega = bonus ? 1.f : a.omega[int64_t(b) * a.om_sb];
  const float u = a.u_res[b];
  block_stats_write<DT, XF, kVW>(rt, red, 0, 0);
  if (!bonus) block_stats_write<DT, XF, kVW>(rd, red, 0, 1);
  __syncthreads();
  float Ct, St, Cd = kRefFloor, Sd = 1.f;
  block_stats_read(red, 0, 0, Ct, St);
  if (!bonus) block_stats_read(red, 0, 1, Cd, Sd);
  ResidCoef k{Ct, 1.f / St, Cd, bonus ? 1.f : 1.f / Sd, omega,
              bonus ? kModeP : (a.resample_mode == 1 ? kModeVanilla : kModeOpt)};
  float R;
  bool writer, trust;
  int token = sample_whole<DT, XF, kVW>(rt, rd, k, u, a.V, sm, R, writer, trust);
  if (draw_needs_fp64(writer, trust, a.exact_draw, &sm.needs64)) {
    const ExactJob job{{t_c, t_u, -INFINITY, (double)Ct}, {d_c, d_u, -INFINITY, (double)Cd}, DT, XF, a.V, a.cfg_scale,
                       a.inv_T, omega, k.mode, nullptr, 0, 0, 0};
    token = exact_draw<kThreadsW>(job, u, R, smx);
    writer = threadIdx.x == 0;
  }
  if (writer) {
    a.next_token[b] = token;
    if (a.resid_mass) a.resid_mass[b] = R;
  }
}

// The same walk for bf16 rows without a logit transform, with a workgroup of 256 threads per
// sequence.  Such rows stay packed in registers (32 words per row and thread), so a thread can
// hold 64 logits of each row plus the next pair in flight, and the fixed cost of a step
// (reductions, accept test, barrier) is spread over four times as many logits per thread as in
// the 1024-thread form: about half the instructions per logit, and up to three sequences share a
// compute unit.  Layout: tiles as in the statistics kernel (vector k*256 + t), so every load is
// contiguous per wave; the draw at the end is the tile -> thread -> element search of the
// long-row kernels.  The logits of x~_i are fetched by one extra load per row, issued with the
// pair, instead of being searched for in the registers.
// The next pair's loads are issued before the current pair is worked on (one unneeded pair per
// sequence).  Fetching a pair only once its predecessor has been accepted, with three workgroups
// per compute unit to hide the latency instead, was measured and is slower at every batch size.
struct SmemT {
  Smem s;
  float red_c[2][2][kWaves];     // [step parity][target / draft][wave]
  float red_s[2][2][kWaves];
  int tok[kMaxLEarly];
  float u[kMaxLEarly];
  float om[kMaxLEarly];
};

__global__ __launch_bounds__(kThreads) void sequence_early_exit_tile_kernel(const KArgs a) {
  constexpr int DT = kDtBF16;
  constexpr bool XF = false;
  constexpr int kE = Vec<DT>::kE, kES = Vec<DT>::kES, kT = Vec<DT>::kT;
  static_assert(RowRegs<DT, XF, kT>::kRaw, "rows stay packed");
  __shared__ SmemT sm;
  __shared__ ExactSmem<kThreads> smx;
  const int b = blockIdx.x, L = a.L, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  struct Slot { uint4 tc[kT], dc[kT]; float tl, dl; };
  // vector k of this thread starts at element (k*256 + tid)*kE; 32-bit offsets from the (uniform)
  // row pointer.  Vectors beyond the end of the row are fetched from its last vector and read
  // as -inf.
  auto fetch = [&](const char* row, int k) -> uint4 {
    const int e = (k * kThreads + tid) * kE;
    return *reinterpret_cast<const uint4*>(row + uint32_t(e < a.V ? e : a.V - kE) * kES);
  };
  auto unpack = [&](RowRegs<DT, XF, kT>& r, const uint4 (&rc)[kT]) {
#pragma unroll
    for (int k = 0; k < kT; ++k) {
      const bool in = (k * kThreads + tid) * kE < a.V;
      r.w[k * 4 + 0] = in ? rc[k].x : 0xFF80FF80u; r.w[k * 4 + 1] = in ? rc[k].y : 0xFF80FF80u;
      r.w[k * 4 + 2] = in ? rc[k].z : 0xFF80FF80u; r.w[k * 4 + 3] = in ? rc[k].w : 0xFF80FF80u;
    }
  };
  // Always the same number of loads, whatever i is (row indices are clamped to the last valid
  // row, whose re-read is harmless), so that the compiler can count the loads in flight.
  auto fetch_vectors = [&](Slot& sl, int i) {
    const int it = min(i, L + a.has_bonus - 1), id = min(i, L - 1);
    const char* tc = row_ptr(a.t, int64_t(b) * a.t_sb + int64_t(it) * a.t_sl, kES);
    const char* dc = row_ptr(a.d, int64_t(b) * a.d_sb + int64_t(id) * a.d_sl, kES);
#pragma unroll
    for (int k = 0; k < kT; ++k) {
      sl.tc[k] = fetch(tc, k);
      sl.dc[k] = fetch(dc, k);
    }
  };
  auto fetch_token_logits = [&](Slot& sl, int i) {
    const int it = min(i, L + a.has_bonus - 1), id = min(i, L - 1);
    const int x = sm.tok[id];
    sl.tl = load_elem<DT>(row_ptr(a.t, int64_t(b) * a.t_sb + int64_t(it) * a.t_sl, kES), x);
    sl.dl = load_elem<DT>(row_ptr(a.d, int64_t(b) * a.d_sb + int64_t(id) * a.d_sl, kES), x);
  };
  auto fetch_pair = [&](Slot& sl, int i) {
    fetch_vectors(sl, i);
    fetch_token_logits(sl, i);
  };
  // the first pair's vectors are requested before anything else: they do not depend on the
  // per-position inputs that are staged in LDS next
  Slot slot;
  fetch_vectors(slot, 0);
  for (int i = tid; i < L; i += kThreads) {
    sm.tok[i] = min(max(a.tokens[int64_t(b) * L + i], 0), a.V - 1);
    sm.u[i] = a.u_acc[int64_t(b) * L + i];
    sm.om[i] = a.omega[int64_t(b) * a.om_sb + i];
  }
  __syncthreads();                                      // tok / u / om are visible
  fetch_token_logits(slot, 0);
  RowRegs<DT, XF, kT> rt, rd;
  rd.clear();

  // statistics of one row over the workgroup: per-wave partials to LDS slot (par, which)
  auto stats_write = [&](const RowRegs<DT, XF, kT>& r, int par, int which) {
    float c, s;
    thread_stats<DT, XF, kT>(r, c, s);
    const float wc = wave_max(c);
    const float ws = wave_sum(s * exp2_fast(c - wc));
    if (lane == 0) { sm.red_c[par][which][wv] = wc; sm.red_s[par][which][wv] = ws; }
  };
  auto stats_read = [&](int par, int which, float& C, float& S) {
    float c[kWaves], sv[kWaves];
#pragma unroll
    for (int w = 0; w < kWaves; ++w) { c[w] = sm.red_c[par][which][w]; sv[w] = sm.red_s[par][which][w]; }
    C = fmaxf(fmaxf(c[0], c[1]), fmaxf(c[2], c[3]));
    S = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) S = __fadd_rn(S, sv[w] * exp2_fast(c[w] - C));
  };

  int j = L;                                            // first rejected position
  float Ct = kRefFloor, St = 1.f, Cd = kRefFloor, Sd = 1.f;
  for (int i = 0; i < L; ++i) {
    unpack(rt, slot.tc);
    unpack(rd, slot.dc);
    const float lt = slot.tl, ld = slot.dl;
    fetch_pair(slot, i + 1);                            // the next pair is in flight during this step
    const int par = i & 1;
    stats_write(rt, par, 0);
    stats_write(rd, par, 1);
    __syncthreads();       // the only barrier of a step: LDS slots alternate with the step parity
    stats_read(par, 0, Ct, St);
    stats_read(par, 1, Cd, Sd);
    // same evaluation of f_i = min{1, omega_i p_i(x~_i) / q_i(x~_i)} as the all-rows path (Eq. relax)
    const double fi = relaxed_accept_prob(lt, ld, Ct, St, Cd, Sd, sm.om[i]);
    if (tid == 0) {
      const int64_t o = int64_t(b) * L + i;
      const float et = __fmaf_rn(lt, kLog2e, -Ct), ed = __fmaf_rn(ld, kLog2e, -Cd);
      if (a.p_tok) a.p_tok[o] = exp2_fast(et) / St;
      if (a.q_tok) a.q_tok[o] = exp2_fast(ed) / Sd;
      if (a.f) a.f[o] = (float)fi;
    }
    if (!((double)sm.u[i] <= fi)) { j = i; break; }             // uniform: every thread sees the same values
  }
  // positions that were never evaluated
  for (int i = j + 1 + tid; i < L; i += kThreads) {
    const int64_t o = int64_t(b) * L + i;
    if (a.p_tok) a.p_tok[o] = NAN;
    if (a.q_tok) a.q_tok[o] = NAN;
    if (a.f) a.f[o] = NAN;
  }
  if (tid == 0) a.accept_len[b] = j;
  const bool bonus = j == L;
  if (bonus) {
    if (!a.has_bonus) {
      if (tid == 0) {
        a.next_token[b] = -1;
        if (a.resid_mass) a.resid_mass[b] = 0.f;
      }
      return;
    }
    // everything was accepted: the slot holds row L+1 of the target (fetched as "pair" L during
    // the last step); its statistics go to the LDS slot of parity L & 1, last used two steps ago
    unpack(rt, slot.tc);
    stats_write(rt, L & 1, 0);
    __syncthreads();
    stats_read(L & 1, 0, Ct, St);
  }
  ResidCoef k{Ct, 1.f / St, Cd, bonus ? 1.f : 1.f / Sd, bonus ? 1.f : sm.om[j],
              bonus ? kModeP : (a.resample_mode == 1 ? kModeVanilla : kModeOpt)};
  float part[kT], R = 0.f;
  bool fell_back = false;
  for (int attempt = 0; attempt < 2; ++attempt) {
    chunk_masses<DT, XF, kT>(rt, rd, k, part, sm.s);
    R = 0.f;
#pragma unroll
    for (int t = 0; t < kT; ++t) R = __fadd_rn(R, sm.s.tile_tot[t]);
    if (R > 0.f || k.mode == kModeP) break;
    k.mode = kModeP;       // no rejection possible at this position: any law is optimal, use p
    fell_back = true;
  }
  bool trust;
  int token = chunk_select<DT, XF, kT>(rt, rd, k, part, __fmul_rn(a.u_res[b], R), sm.s, trust);
  token = min(max(token, 0), a.V - 1);
  // the fp32 draw stands unless a level fell back, the law is light, or p had to take the place of
  // a law without fp32 mass
  if (!trust || fell_back || (k.mode != kModeP && R < kSafeMass) || a.exact_draw) {
    const int jt = bonus ? L : j;
    const int64_t ot = int64_t(b) * a.t_sb + int64_t(jt) * a.t_sl, od = int64_t(b) * a.d_sb + int64_t(min(jt, L - 1)) * a.d_sl;
    const ExactJob job{{row_ptr(a.t, ot, kES), nullptr, -INFINITY, (double)Ct},
                       {bonus ? nullptr : row_ptr(a.d, od, kES), nullptr, -INFINITY, (double)Cd},
                       DT, XF, a.V, 1.f, 1.f, k.omega, fell_back ? (a.resample_mode == 1 ? kModeVanilla : kModeOpt) : k.mode,
                       nullptr, 0, 0, 0};
    token = exact_draw<kThreads>(job, a.u_res[b], R, smx);
  }
  if (tid == 0) {
    a.next_token[b] = token;
    if (a.resid_mass) a.resid_mass[b] = R;
  }
}

}  // namespace csd
