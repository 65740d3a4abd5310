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
// sequence), sequence_kernel<kMasses> (mass of every 8192-logit chunk of the sampled rows,
// streaming) and sequence_kernel<kSelect> (pick the chunk that holds u*R, re-read it, inverse
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

// ============================================================================ kernel 1
// Softmax statistics of one chunk of one row.  Rows are numbered: target rows first
// (b*(L+has_bonus) + i), then draft rows (rows_t + b*L + i).
struct RowRef {
  int r, b, i;
  bool is_draft;
  const char* cond;
  const char* uncond;
};
// Which row a workgroup of a statistics kernel works on.  G3: the grid is (chunks, rows of one
// sequence -- target rows, then draft rows --, sequences), so no division is needed; otherwise
// the row number is `lin` (used when a grid dimension would exceed 65535).
template <int DT, bool G3> __device__ __forceinline__ RowRef row_ref(const KArgs& a, int lin) {
  constexpr int kES = Vec<DT>::kES;
  RowRef o;
  const int per_t = a.L + a.has_bonus;
  if (G3) {
    o.b = blockIdx.z;
    o.is_draft = (int)blockIdx.y >= per_t;
    o.i = o.is_draft ? blockIdx.y - per_t : blockIdx.y;
    o.r = o.is_draft ? a.rows_t + o.b * a.L + o.i : o.b * per_t + o.i;
  } else {
    o.r = lin;
    o.is_draft = lin >= a.rows_t;
    const int rr = o.is_draft ? lin - a.rows_t : lin;
    const int per = o.is_draft ? a.L : per_t;
    o.b = rr / per;
    o.i = rr - o.b * per;
  }
  const int64_t off = o.is_draft ? int64_t(o.b) * a.d_sb + int64_t(o.i) * a.d_sl
                                 : int64_t(o.b) * a.t_sb + int64_t(o.i) * a.t_sl;
  o.cond = row_ptr(o.is_draft ? a.d : a.t, off, kES);
  o.uncond = row_ptr(o.is_draft ? a.du : a.tu, off, kES);
  return o;
}

// The draft token x~_i of a row (or -1), fetched with a per-lane load: a load from an address
// the compiler can prove uniform would go through the scalar cache and the wait for it would
// also hold back the chunk's vector loads that follow in program order.
__device__ __forceinline__ int load_draft_token(const KArgs& a, const RowRef& rw) {
  if (a.tokens == nullptr || rw.i >= a.L) return -1;
  int z = 0;
  asm volatile("" : "+v"(z));
  return a.tokens[int64_t(rw.b) * a.L + rw.i + z];
}

__device__ __forceinline__ float token_logit_any(int dt, const char* cond, const char* uncond, int x, bool xf,
                                                 float s, float inv_T, float thr) {
  float lc = dt == kDtBF16 ? load_elem<kDtBF16>(cond, x) : load_elem<kDtF32>(cond, x);
  if (!xf) return lc;
  float lu = 0.f;
  if (uncond) lu = dt == kDtBF16 ? load_elem<kDtBF16>(uncond, x) : load_elem<kDtF32>(uncond, x);
  const float l = transform_logit(lc, lu, uncond != nullptr, s, inv_T);
  return l >= thr ? l : -INFINITY;
}

// Eq. f_lantern for position pos = (b, i), by one wave: gathers the k neighbour logits of x~_i,
// scans their weights 2^((l_n - l_x) log2e) and leaves agg = (sum over the set) / p_i(x~_i) >= 1
// and the member count in the workspace (plus the optional count output).  Needs no row
// statistics; under top-k it needs the target row's threshold thr (-inf: no truncation).
__device__ __forceinline__ void lantern_agg_position(const KArgs& a, int pos, int dt, bool xf, float thr) {
  const int lane = threadIdx.x & 63;
  const int b = pos / a.L, i = pos - b * a.L;
  const int es = dt == kDtBF16 ? 2 : 4;
  const int64_t off = int64_t(b) * a.t_sb + int64_t(i) * a.t_sl;
  const char* cond = row_ptr(a.t, off, es);
  const char* uncond = row_ptr(a.tu, off, es);
  const int x = min(max(a.tokens[pos], 0), a.V - 1);
  // the (transformed, masked) logit of x~_i: the same value the statistics kernel leaves in
  // tok_logit, formed here so that this does not have to wait for that kernel
  const float lx = token_logit_any(dt, cond, uncond, x, xf, a.cfg_scale, a.inv_T, thr);
  const int32_t* row = a.nbr + int64_t(x) * a.lan_k;
  float cum = 0.f;
  int m = 0;
  if (lx > -INFINITY) {                       // p(x~) = 0 admits no neighbour: nothing is below 0
    for (int j0 = 0; j0 < a.lan_k; j0 += 64) {
      const int j = j0 + lane;
      const int n = j < a.lan_k ? row[j] : -1;
      const bool valid = n >= 0 && n < a.V && n != x;
      const float ln = valid ? token_logit_any(dt, cond, uncond, n, xf, a.cfg_scale, a.inv_T, thr) : -INFINITY;
      const float w = valid ? exp2_fast(__fmul_rn(__fsub_rn(ln, lx), kLog2e)) : 0.f;
      const float incl = __fadd_rn(cum, wave_scan_incl(w));
      const unsigned long long bv = __ballot(valid);
      const unsigned long long bf = __ballot(valid && !(incl < a.lan_lambda));
      if (bf) {                                // the first neighbour that does not fit ends the set
        const int fl = __ffsll((long long)bf) - 1;
        m += __popcll(bv & ((1ull << fl) - 1ull));
        // the running sum before lane fl: weights of skipped lanes are zero, so it is the sum
        // over the members taken so far
        if (fl > 0) cum = lane_f(incl, fl - 1);
        break;
      }
      m += __popcll(bv);
      cum = lane_f(incl, 63);
    }
  }
  if (lane == 0) {
    a.lan_omega[pos] = __fadd_rn(1.f, cum);
    a.lan_count[pos] = m;
    if (a.count_out) a.count_out[pos] = m;
  }
}

// LAN: cool_sd_verify_lantern without top-k appends workgroups to this launch that do the
// neighbour aggregation (one wave per position) instead of statistics -- it needs nothing the
// statistics produce, so it costs no launch of its own.  They are the grid's z-slices from B on
// (G3) or the workgroups after the last chunk.
template <int DT, bool XF, int AL, int NT, bool G3, bool LAN = false>
__global__ __launch_bounds__(kThreads, 3) void row_stats_kernel(const KArgs a) {
  constexpr int kE = Vec<DT>::kE;
  __shared__ float red_c[kWaves], red_s[kWaves];
  const int C1 = a.c1;
  if constexpr (LAN) {
    const int64_t extra = G3 ? (int64_t(blockIdx.z) - a.B) * (int64_t(gridDim.y) * gridDim.x) + int64_t(blockIdx.y) * gridDim.x + blockIdx.x
                             : int64_t(blockIdx.x) - (int64_t(a.rows_t) + a.rows_d) * C1;
    if (G3 ? (int)blockIdx.z >= a.B : extra >= 0) {
      const int64_t pos = extra * kWaves + (threadIdx.x >> 6);
      if (pos < int64_t(a.B) * a.L) lantern_agg_position(a, (int)pos, DT, XF, -INFINITY);
      return;
    }
  }
  const int lin = G3 ? 0 : blockIdx.x / C1, c = G3 ? blockIdx.x : blockIdx.x - lin * C1;
  const RowRef rw = row_ref<DT, G3>(a, lin);
  const int r = rw.r;
  const int64_t base = int64_t(c) * (NT * kThreads * kE);

  // rows longer than one workgroup under top-k: the threshold was selected by the radix passes
  float thr = -INFINITY;
  if constexpr (XF) {
    if (a.top_k > 0) thr = a.thr[r];
  }
  RowRegs<DT, XF, NT> x;
  load_chunk<DT, XF, AL, NT>(x, rw.cond, rw.uncond, base, a.V, a.cfg_scale, a.inv_T, thr);
  int tok = load_draft_token(a, rw);     // after the chunk's loads in program order, used after them
  // the (transformed) logit of x~_i for the accept test of the next kernel, taken from the
  // registers of the thread that holds it: element e of vector (tile k, thread t) is token
  // base + (k*256 + t)*kE + e
  if (tok >= 0) {
    tok = min(tok, a.V - 1);
    const int64_t rel = int64_t(tok) - base;
    if (rel >= 0 && rel < NT * kThreads * kE) {
      const int vec = int(rel) / kE, e = int(rel) - vec * kE;
      if ((vec & (kThreads - 1)) == (int)threadIdx.x) {
        const int k = vec / kThreads;
        float l = 0.f;
#pragma unroll
        for (int kk = 0; kk < NT; ++kk) {
#pragma unroll
          for (int j = 0; j < kE; ++j) l = (kk == k && j == e) ? x.get(kk, j) : l;
        }
        a.tok_logit[r] = l;
      }
    }
  }
  float ct, st;
  thread_stats<DT, XF, NT>(x, ct, st);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const float wc = wave_max(ct);
  const float ws = wave_sum(st * exp2_fast(ct - wc));     // exact power-of-two rescale
  if (lane == 0) { red_c[wv] = wc; red_s[wv] = ws; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const float C = fmaxf(fmaxf(red_c[0], red_c[1]), fmaxf(red_c[2], red_c[3]));
    float S = red_s[0] * exp2_fast(red_c[0] - C);
    S = __fadd_rn(S, red_s[1] * exp2_fast(red_c[1] - C));
    S = __fadd_rn(S, red_s[2] * exp2_fast(red_c[2] - C));
    S = __fadd_rn(S, red_s[3] * exp2_fast(red_c[3] - C));
    a.part[int64_t(r) * C1 + c] = make_float2(C, S);
  }
}

// Statistics of whole rows under top-k truncation: one workgroup of TPB threads per row,
// ROW / TPB transformed logits per thread in registers (ROW = 16384 with 512 threads, or 65536
// with 1024 threads for vocabularies up to 64K).  The k-th largest value of the row is selected
// first (topk.h); the softmax statistics are then taken over the entries >= that threshold,
// against the reference exponent of the row maximum (always kept).  Writes the row's threshold,
// its statistics -- one pair per row, or for the long form one pair per 8192 logits, the layout
// the sampling kernels of long rows expect -- and the masked logit of x~_i.  The work per row is
// a chain of short block-wide phases bound by instruction issue, so the code is kept lean and
// the row is spread over enough threads that several rows fit a compute unit.
constexpr int kThreadsK = 512;
constexpr int kRowMid = 4 * kChunk;      // longest row the one-workgroup form takes (1024 threads)
template <int DT, int AL, int TPB, int GD, bool G3, int ROW, bool LAN = false>
__global__ __launch_bounds__(TPB, ROW == kChunk ? 6 : 4) void row_stats_topk_kernel(const KArgs a) {
  constexpr int kE = Vec<DT>::kE;
  constexpr int kVW = ROW / (TPB * kE);                // vectors per thread
  constexpr int kW = TPB / 64;
  constexpr int kSub = ROW == kChunk ? 1 : ROW / 8192; // statistics pairs per row
  constexpr int kTS = kVW / kSub;                      // this thread's vectors per pair: tile k covers
                                                       // TPB*kE consecutive logits, 8192 / (TPB*kE) tiles per pair
  __shared__ TopkSmem<TPB> ts;
  __shared__ float red_s[kSub][kW];
  const RowRef rw = row_ref<DT, G3>(a, blockIdx.x);
  const int r = rw.r;
  topk_prepare(ts);                                     // the barrier inside topk_threshold orders it
  RowRegs<DT, true, kVW> x;
  // vector k of thread t is vector k*TPB + t of the row
  load_chunk<DT, true, AL, kVW, TPB, 1, 4, GD>(x, rw.cond, rw.uncond, 0, a.V, a.cfg_scale, a.inv_T, -INFINITY);
  // the raw logits of x~_i, requested now and used at the very end
  int tok = load_draft_token(a, rw);
  float tok_c = 0.f, tok_u = 0.f;
  if (tok >= 0 && threadIdx.x == 0) {
    tok = min(tok, a.V - 1);
    tok_c = load_elem<DT>(rw.cond, tok);
    if (rw.uncond) tok_u = load_elem<DT>(rw.uncond, tok);
  }
  float row_max;
  const float thr = topk_threshold<kVW * kE, TPB>(x.w, a.top_k, ts, row_max);
  const float c = fmaxf(ceilf(row_max * kLog2e), kRefFloor);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
  for (int sub = 0; sub < kSub; ++sub) {
    float s = 0.f;
#pragma unroll
    for (int n = sub * kTS * kE; n < (sub + 1) * kTS * kE; ++n) {
      const float l = __uint_as_float(x.w[n]);
      const float e = exp2_fast(__fmaf_rn(l, kLog2e, -c));
      s += (l >= thr) ? e : 0.f;
    }
    s = wave_sum(s);
    if (lane == 0) red_s[sub][wv] = s;
  }
  __syncthreads();
  if ((int)threadIdx.x < kSub && (int)threadIdx.x < a.c1) {
    float S = red_s[threadIdx.x][0];
#pragma unroll
    for (int w = 1; w < kW; ++w) S = __fadd_rn(S, red_s[threadIdx.x][w]);
    a.part[int64_t(r) * a.c1 + threadIdx.x] = make_float2(c, S);
  }
  if (threadIdx.x == 0) {
    a.thr[r] = thr;
    if (tok >= 0) {
      const float l = transform_logit(tok_c, tok_u, rw.uncond != nullptr, a.cfg_scale, a.inv_T);
      a.tok_logit[r] = (l >= thr) ? l : -INFINITY;
    }
  }
  if constexpr (LAN) {
    // cool_sd_verify_lantern: the workgroup of a target row has that row's threshold, which is all
    // the neighbour aggregation of its position needs; its first wave does it here instead of in
    // a launch of its own
    if (!rw.is_draft && rw.i < a.L && threadIdx.x < 64) lantern_agg_position(a, rw.b * a.L + rw.i, DT, true, thr);
  }
}

// The drafting stage's draw under top-k truncation, in ONE launch: cool_sd_resample without a draft
// on rows of at most 16384 logits.  Same selection of the threshold as row_stats_topk_kernel; the
// kept entries' weights 2^(l log2e - c) then stay in the registers and x~ is drawn from them by
// the tile -> thread -> element search (tile k of the row is the TPB*kE consecutive logits from
// k*TPB*kE on; thread t owns vector t of each tile), each level "first positive-mass entry whose
// inclusive sum exceeds the remainder, else the last positive-mass entry".
template <int DT, int AL, int GD>
__global__ __launch_bounds__(kThreadsK) void resample_topk_kernel(const KArgs a) {
  constexpr int TPB = kThreadsK, kE = Vec<DT>::kE, kES = Vec<DT>::kES;
  constexpr int kVW = kChunk / (TPB * kE);             // tiles: 4 (bf16) / 8 (fp32)
  constexpr int kW = TPB / 64;
  static_assert(kVW <= 8, "tile_part holds up to 8 tiles");
  __shared__ TopkSmem<TPB> ts;
  __shared__ float tile_part[kW][8];
  __shared__ float scan_tot[kW];
  __shared__ int pick_first[kW], pick_last[kW];
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  topk_prepare(ts);
  RowRegs<DT, true, kVW> x;
  load_chunk<DT, true, AL, kVW, TPB, 1, 4, GD>(x, row_ptr(a.t, int64_t(b) * a.t_sb, kES), row_ptr(a.tu, int64_t(b) * a.t_sb, kES),
                                                0, a.V, a.cfg_scale, a.inv_T, -INFINITY);
  const float u = a.u_res[b];
  float row_max;
  const float thr = topk_threshold<kVW * kE, TPB>(x.w, a.top_k, ts, row_max);
  const float c = fmaxf(ceilf(row_max * kLog2e), kRefFloor);
  // weights of the kept entries, in place of the logits; per-tile partial sums
  float part[kVW];
#pragma unroll
  for (int k = 0; k < kVW; ++k) {
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < kE; ++j) {
      const float l = __uint_as_float(x.w[k * kE + j]);
      const float e = exp2_fast(__fmaf_rn(l, kLog2e, -c));
      const float m = (l >= thr) ? e : 0.f;
      x.w[k * kE + j] = __float_as_uint(m);
      acc = __fadd_rn(acc, m);
    }
    part[k] = acc;
  }
#pragma unroll
  for (int k = 0; k < kVW; ++k) {
    const float v = wave_sum(part[k]);
    if (lane == 0) tile_part[wv][k] = v;
  }
  __syncthreads();
  // level 1: tile
  float T[kVW], R = 0.f;
#pragma unroll
  for (int k = 0; k < kVW; ++k) {
    float tsum = 0.f;
#pragma unroll
    for (int w = 0; w < kW; ++w) tsum = __fadd_rn(tsum, tile_part[w][k]);
    T[k] = tsum;
    R = __fadd_rn(R, tsum);
  }
  const float v = __fmul_rn(u, R);
  int ks = -1, klast = -1;
  float base = 0.f, base_last = 0.f, cum = 0.f;
#pragma unroll
  for (int k = 0; k < kVW; ++k) {
    if (T[k] > 0.f) {
      if (ks < 0 && __fadd_rn(cum, T[k]) > v) { ks = k; base = cum; }
      klast = k; base_last = cum;
    }
    cum = __fadd_rn(cum, T[k]);
  }
  if (ks < 0) { ks = klast; base = base_last; }
  if (ks < 0) {            // a row without any finite logit: outside the contract, answer token 0
    if (tid == 0) { a.next_token[b] = 0; if (a.resid_mass) a.resid_mass[b] = 0.f; }
    return;
  }
  const float v2 = v - base;
  // level 2: thread
  float my = 0.f;
#pragma unroll
  for (int k = 0; k < kVW; ++k) my = (k == ks) ? part[k] : my;
  const float incl_w = wave_scan_incl(my);
  const float excl_w = wave_prev_lane(incl_w);
  if (lane == 63) scan_tot[wv] = incl_w;
  __syncthreads();
  float woff = 0.f;
#pragma unroll
  for (int w = 0; w < kW; ++w) woff = (w < wv) ? __fadd_rn(woff, scan_tot[w]) : woff;
  const float incl = __fadd_rn(woff, incl_w), excl = __fadd_rn(woff, lane == 0 ? 0.f : excl_w);
  const bool pos = my > 0.f;
  const bool hit = pos && (incl > v2);
  const unsigned long long bh = __ballot(hit), bp = __ballot(pos);
  if (lane == 0) {
    pick_first[wv] = bh ? (wv * 64 + __ffsll((long long)bh) - 1) : 0x7fffffff;
    pick_last[wv] = bp ? (wv * 64 + 63 - __clzll((long long)bp)) : -1;
  }
  __syncthreads();
  int win = 0x7fffffff, last_pos = -1;
#pragma unroll
  for (int w = 0; w < kW; ++w) { win = min(win, pick_first[w]); last_pos = max(last_pos, pick_last[w]); }
  if (win == 0x7fffffff) win = last_pos;
  // level 3: element, by the winning thread
  if (tid == win) {
    const float v3 = v2 - excl;
    int found = -1, last = 0;
    float run = 0.f;
#pragma unroll
    for (int j = 0; j < kE; ++j) {
      float m = 0.f;
#pragma unroll
      for (int k = 0; k < kVW; ++k) m = (k == ks) ? __uint_as_float(x.w[k * kE + j]) : m;
      if (m > 0.f) {
        last = j;
        run = __fadd_rn(run, m);
        if (found < 0 && run > v3) found = j;
      }
    }
    if (found < 0) found = last;
    a.next_token[b] = min((ks * TPB + win) * kE + found, a.V - 1);
    if (a.resid_mass) a.resid_mass[b] = 1.f;             // the law is p itself
  }
}

// ---------------------------------------------------------------------------- top-k, long rows
// Rows that do not fit one workgroup: the k-th largest transformed logit is found by a radix
// select on the order-preserving 32-bit key in three passes of 11, 11 and 10 bits.  A pass is two
// launches: every chunk's workgroup counts, in LDS, the digit of its values whose higher bits
// match what earlier passes fixed and adds the non-empty buckets to the row's histogram in the
// workspace (integer atomics: the sums do not depend on the order); then one workgroup per row
// walks the histogram from the top, fixes the digit that holds the k-th largest and clears the
// histogram for the next pass.  After the third pass the key is exact, ties included, and the
// ordinary statistics kernel masks with its value.  Elements beyond the end of a row count as
// -inf: they are the smallest keys and never change which value is the k-th largest among at
// least k real ones.
constexpr int kRadixBuckets = 2048;
__device__ __forceinline__ int radix_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ int radix_bits(int pass) { return pass == 2 ? 10 : 11; }

template <int DT, int AL, int NT, bool G3>
__global__ __launch_bounds__(kThreads) void topk_radix_hist_kernel(const KArgs a, int pass) {
  constexpr int kE = Vec<DT>::kE;
  __shared__ uint32_t hist[kRadixBuckets];
  const int C1 = a.c1;
  const int lin = G3 ? 0 : blockIdx.x / C1, c = G3 ? blockIdx.x : blockIdx.x - lin * C1;
  const RowRef rw = row_ref<DT, G3>(a, lin);
  const int r = rw.r;
  for (int i = threadIdx.x; i < kRadixBuckets; i += kThreads) hist[i] = 0u;
  RowRegs<DT, true, NT> x;
  load_chunk<DT, true, AL, NT>(x, rw.cond, rw.uncond, int64_t(c) * (NT * kThreads * kE), a.V, a.cfg_scale, a.inv_T,
                               -INFINITY);
  const int shift = radix_shift(pass), bits = radix_bits(pass);
  const uint32_t prefix = pass > 0 ? a.rk_state[2 * r] : 0u;
  const int hshift = shift + bits;                        // bits above the digit, fixed by earlier passes
  __syncthreads();
#pragma unroll
  for (int n = 0; n < NT * kE; ++n) {
    const uint32_t key = order_key(__uint_as_float(x.w[n]));
    const bool match = pass == 0 || (key >> hshift) == (prefix >> hshift);
    if (match) atomicAdd(&hist[(key >> shift) & ((1u << bits) - 1u)], 1u);
  }
  __syncthreads();
  for (int i = threadIdx.x; i < kRadixBuckets; i += kThreads) {
    const uint32_t h = hist[i];
    if (h) atomicAdd(&a.rk_hist[int64_t(r) * kRadixBuckets + i], h);
  }
}

// One workgroup per row: the digit of this pass that holds the k-th largest key.  Thread t owns
// the eight buckets 2047 - 8t .. 2040 - 8t, so that ascending thread order is descending key order.
__global__ __launch_bounds__(kThreads) void topk_radix_select_kernel(const KArgs a, int pass) {
  __shared__ uint32_t wave_tot[kWaves];
  const int r = blockIdx.x;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  uint32_t* hist = a.rk_hist + int64_t(r) * kRadixBuckets;
  const uint32_t k_rem = pass == 0 ? (uint32_t)a.top_k : a.rk_state[2 * r + 1];
  const uint32_t prefix = pass == 0 ? 0u : a.rk_state[2 * r];
  uint32_t h[8], local = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const int bkt = kRadixBuckets - 1 - (threadIdx.x * 8 + j);
    h[j] = hist[bkt];
    hist[bkt] = 0u;                                       // ready for the next pass / the next call
    local += h[j];
  }
  const uint32_t incl = wave_scan_incl_u32(local);
  if (lane == 63) wave_tot[wv] = incl;
  __syncthreads();
  uint32_t before = incl - local;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) before += (w < wv) ? wave_tot[w] : 0u;
  if (before < k_rem && k_rem <= before + local) {        // exactly one thread
    uint32_t cum = before;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (cum < k_rem && k_rem <= cum + h[j]) {
        const uint32_t digit = (uint32_t)(kRadixBuckets - 1 - (threadIdx.x * 8 + j));
        const uint32_t np = prefix | (digit << radix_shift(pass));
        a.rk_state[2 * r] = np;
        a.rk_state[2 * r + 1] = k_rem - cum;
        if (pass == 2) a.thr[r] = key_value(np);
      }
      cum += h[j];
    }
  }
}

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
__global__ __launch_bounds__(kThreads) void combine_rows_kernel(const KArgs a) {
  const int r = blockIdx.x * kWaves + (threadIdx.x >> 6);
  if (r >= a.rows_t + a.rows_d) return;
  combine_row_wave(a, r);
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
template <int DT, bool XF, int kT, bool LAN = false>
__device__ __forceinline__ int chunk_select(const RowRegs<DT, XF, kT>& rt, const RowRegs<DT, XF, kT>& rd,
                                            const ResidCoef& k, const float (&part)[kT],
                                            float v, Smem& sm, const LanPatch lp = LanPatch{0u, -1, 1.f}) {
  constexpr int kE = Vec<DT>::kE;
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
          const float r = tile_elem<DT, XF, kT, LAN>(rt, rd, k, lp, t, j);
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
  // exponents of p(x~) and q(x~) in base-2 units; the ratio p/q is formed from their
  // difference so that it survives when both probabilities underflow fp32
  const float et = __fmaf_rn(lt, kLog2e, -Ct), ed = __fmaf_rn(ld, kLog2e, -Cd);
  const float ratio = __fmul_rn(exp2_fast(__fsub_rn(et, ed)), Sd / St);
  // f = min{1, omega p/q}; a token the draft excludes (q = 0) has f = 1, also at 0/0
  const float fi = (ld == -INFINITY) ? 1.f : ((omega > 0.f) ? fminf(1.f, __fmul_rn(omega, ratio)) : 0.f);
  if (emit && has_draft) {
    const int64_t o = int64_t(b) * a.L + i;
    // aggregated probability of the neighbour set (Eq. p_lantern at x~_i): p_i(x~_i) times agg,
    // which the LANTERN-style call passes as omega_i
    if (a.p_agg_out) a.p_agg_out[o] = __fmul_rn(exp2_fast(et) / St, omega);
    if (a.p_tok) a.p_tok[o] = exp2_fast(et) / St;
    if (a.q_tok) a.q_tok[o] = exp2_fast(ed) / Sd;
    if (a.f) a.f[o] = fi;
  }
  if (!has_draft) { Cd = kRefFloor; Sd = 0.f; }         // the bonus row stands alone
  return has_draft && !(u <= fi);
}

// Accept test at every position of sequence b (Eq. relax) and tau = first rejection (Algorithm 1)
// by the TPB threads of a workgroup.  Leaves the combined statistics (Ct, St, Cd, Sd) of the row
// that will be sampled from -- position tau+1, or the bonus row L+1 -- in *rowstat and returns tau.
// With `emit` it also writes accept_len and the per-position diagnostics.
template <int DT, bool XF, int TPB>
__device__ __forceinline__ int find_tau(const KArgs& a, int b, bool emit, int* pick /*[TPB/64]*/, float4* rowstat) {
  const int rps = a.L + a.has_bonus;
  if (rps <= 64) {
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
};

// Middle kernel of the several-chunk path: one workgroup per sequence finds tau and leaves
// accept_len[b] and the sampled row's statistics for the sampling kernel.
template <int DT, bool XF>
__global__ __launch_bounds__(kThreadsW) void accept_kernel(const KArgs a) {
  __shared__ SmemW sm;
  const int b = blockIdx.x;
  if (a.accept_combines) {
    // rows of many statistics chunks: combine the chunks of this sequence's rows first, one wave
    // per row (what combine_rows_kernel does for all rows), then read them back below.  Sixteen
    // waves, so that a window of eight positions is one or two rows per wave: each row is a
    // memory round trip of its own.
    const int rps = a.L + a.has_bonus;
    for (int q = threadIdx.x >> 6; q < rps + a.L; q += kWavesW)
      combine_row_wave(a, q < rps ? b * rps + q : a.rows_t + b * a.L + (q - rps));
    __syncthreads();          // the rows' statistics are visible to the whole workgroup
  }
  const int j = find_tau<DT, XF, kThreadsW>(a, b, true, sm.pick, &sm.rowstat);
  if (threadIdx.x == 0) a.seq_stat[b] = sm.rowstat;
  (void)j;
}

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
template <int DT, bool XF, int kVW, bool LAN = false>
__device__ __forceinline__ int sample_whole(const RowRegs<DT, XF, kVW>& rt, const RowRegs<DT, XF, kVW>& rd,
                                            ResidCoef k, float u, int V, SmemW& sm, float& R, bool& writer,
                                            const LanPatch lp = LanPatch{0u, -1, 1.f}) {
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
    if (R > 0.f || k.mode == kModeP) break;
    k.mode = kModeP;   // no rejection possible at this position: any law is optimal, use p
  }

  // thread: first with positive mass whose inclusive sum exceeds u*R, else the last with mass
  const float v = __fmul_rn(u, R);
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
  if (win == 0x7fffffff) win = last_pos;
  writer = win >= 0 ? (int)threadIdx.x == win : threadIdx.x == 0;   // a row without any mass: token 0
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
    if (vs < 0) { vs = vlast; vbase = vbase_last; }
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
    if (found < 0) found = last;
    token = (win * kVW + vs) * kE + found;
  }
  return token >= V ? V - 1 : token;
}

template <int DT, bool XF, bool AL, bool LAN>
__global__ __launch_bounds__(kThreadsW) void sequence_whole_kernel(const KArgs a) {
  constexpr int kE = Vec<DT>::kE, kES = Vec<DT>::kES;
  constexpr int kVW = kChunk / (kThreadsW * kE);       // vectors per thread: 2 (bf16) / 4 (fp32)
  __shared__ SmemW sm;
  const int b = blockIdx.x;
  const int rps = a.L + a.has_bonus;
  const bool masked = XF && a.top_k > 0;


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
  bool writer;
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
    }
    token = sample_whole<DT, XF, kVW, true>(rt, rd, k, a.u_res[b], a.V, sm, R, writer, lp);
  } else {
    token = sample_whole<DT, XF, kVW>(rt, rd, k, a.u_res[b], a.V, sm, R, writer);
  }
  if (writer) {
    a.next_token[b] = token;
    if (a.resid_mass) a.resid_mass[b] = R;
  }
}

// ============================================================================ neighbour aggregation
// Eq. f_lantern: the acceptance probability of x~_i uses the probability of its neighbour set
// A(x~_i) = {x~_i} + the longest prefix of its neighbour list (nearest first) whose summed
// probability stays below lambda p_i(x~_i).  Relative to p_i(x~_i) the members weigh
// 2^((l_n - l_x) log2e), which needs no row statistics, so one wave per position gathers the k
// neighbour logits, scans their weights and leaves agg = sum over A / p_i(x~_i) >= 1 where the
// accept test reads its relaxation parameter: Eq. f_lantern is Eq. relax with omega_i = agg.
// Also writes the number of members (for Eq. g_lantern) and the optional outputs.
__global__ __launch_bounds__(kThreads) void lantern_agg_kernel(const KArgs a, int dt, int xf) {
  const int pos = blockIdx.x * kWaves + (threadIdx.x >> 6);       // (b, i)
  if (pos >= a.B * a.L) return;
  const int b = pos / a.L, rt_ = b * (a.L + a.has_bonus) + (pos - b * a.L);
  lantern_agg_position(a, pos, dt, xf != 0, (xf && a.top_k > 0) ? a.thr[rt_] : -INFINITY);
}

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
  const int b = blockIdx.x, L = a.L, tid = threadIdx.x;
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
    const float et = __fmaf_rn(lt, kLog2e, -Ct), ed = __fmaf_rn(ld, kLog2e, -Cd);
    const float ratio = __fmul_rn(exp2_fast(__fsub_rn(et, ed)), Sd / St);
    const float omega = sm.om[i];
    const float fi = (ld == -INFINITY) ? 1.f : ((omega > 0.f) ? fminf(1.f, __fmul_rn(omega, ratio)) : 0.f);
    if (tid == 0) {
      const int64_t o = int64_t(b) * L + i;
      if (a.p_tok) a.p_tok[o] = exp2_fast(et) / St;
      if (a.q_tok) a.q_tok[o] = exp2_fast(ed) / Sd;
      if (a.f) a.f[o] = fi;
    }
    return !(sm.u[i] <= fi);                            // uniform: every thread sees the same values
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
  bool writer;
  const int token = sample_whole<DT, XF, kVW>(rt, rd, k, a.u_res[b], a.V, sm.w, R, writer);
  if (writer) {
    a.next_token[b] = token;
    if (a.resid_mass) a.resid_mass[b] = R;
  }
}

// cool_sd_resample on rows of at most 16384 logits without top-k, in ONE launch: a workgroup of
// 1024 threads holds the row pair (or the single row when no draft is given), forms its softmax
// statistics block-wide and draws the token from the registers.  The drafting loop calls this once
// per drafted token, so its latency (one launch instead of two) is what matters.
template <int DT, bool XF, bool AL>
__global__ __launch_bounds__(kThreadsW) void resample_whole_kernel(const KArgs a) {
  constexpr int kE = Vec<DT>::kE, kES = Vec<DT>::kES;
  constexpr int kVW = kChunk / (kThreadsW * kE);
  __shared__ SmemW sm;
  __shared__ RedW red;
  const int b = blockIdx.x;
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
  bool writer;
  const int token = sample_whole<DT, XF, kVW>(rt, rd, k, u, a.V, sm, R, writer);
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
    const float et = __fmaf_rn(lt, kLog2e, -Ct), ed = __fmaf_rn(ld, kLog2e, -Cd);
    const float ratio = __fmul_rn(exp2_fast(__fsub_rn(et, ed)), Sd / St);
    const float omega = sm.om[i];
    const float fi = (ld == -INFINITY) ? 1.f : ((omega > 0.f) ? fminf(1.f, __fmul_rn(omega, ratio)) : 0.f);
    if (tid == 0) {
      const int64_t o = int64_t(b) * L + i;
      if (a.p_tok) a.p_tok[o] = exp2_fast(et) / St;
      if (a.q_tok) a.q_tok[o] = exp2_fast(ed) / Sd;
      if (a.f) a.f[o] = fi;
    }
    if (!(sm.u[i] <= fi)) { j = i; break; }             // uniform: every thread sees the same values
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
  for (int attempt = 0; attempt < 2; ++attempt) {
    chunk_masses<DT, XF, kT>(rt, rd, k, part, sm.s);
    R = 0.f;
#pragma unroll
    for (int t = 0; t < kT; ++t) R = __fadd_rn(R, sm.s.tile_tot[t]);
    if (R > 0.f || k.mode == kModeP) break;
    k.mode = kModeP;       // no rejection possible at this position: any law is optimal, use p
  }
  const int off = chunk_select<DT, XF, kT>(rt, rd, k, part, __fmul_rn(a.u_res[b], R), sm.s);
  if (tid == 0) {
    a.next_token[b] = min(max(off, 0), a.V - 1);
    if (a.resid_mass) a.resid_mass[b] = R;
  }
}

// ============================================================================ kernel 2, long rows
// Long rows (more than 16384 logits): the draw x_{tau+1} from the resampling law of the sampled
// row (Eq. opt_G / Eq. g_tsd / p_{L+1}) in two launches.  STAGE selects what one launch does:
//   kMasses  grid = B x C.  Rows of C chunks: workgroup (b, c) writes the mass of chunk c.
//   kSelect  grid = B.      Rows of C chunks: pick the chunk that holds u*R, load it, inverse CDF.
enum { kMasses = 1, kSelect = 2 };

template <int DT, bool XF, bool AL, int kT, int STAGE, bool LAN>
__global__ __launch_bounds__(kThreads) void sequence_kernel(const KArgs a) {
  constexpr int kES = Vec<DT>::kES;
  constexpr int kChunk2 = kT * kThreads * Vec<DT>::kE;   // logits per sampling chunk
  __shared__ Smem sm;
  const int C = a.nchunks;
  const int b = (STAGE == kMasses) ? blockIdx.x / C : blockIdx.x;
  const int c = (STAGE == kMasses) ? blockIdx.x - b * C : 0;
  const int rps = a.L + a.has_bonus;
  const bool masked = XF && a.top_k > 0;

  int j = 0;
  if (!a.resample_only) {
    j = a.accept_len[b];
    if (j >= a.L && !a.has_bonus) {
      if (STAGE != kMasses && threadIdx.x == 0) {
        a.next_token[b] = -1;
        if (a.resid_mass) a.resid_mass[b] = 0.f;
      }
      return;
    }
  }

  // ---- the row that is sampled from: position tau+1, or the bonus row (Algorithm 1)
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
  // the statistics of the sampled row are the same for every thread: read straight from the
  // workspace (a scalar load that is in flight while the chunk's vector loads are issued)
  const float4 rs = a.resample_only ? sm.rowstat : a.seq_stat[b];
  const char* t_c = row_ptr(a.t, int64_t(b) * a.t_sb + int64_t(j) * a.t_sl, kES);
  const char* t_u = row_ptr(a.tu, int64_t(b) * a.t_sb + int64_t(j) * a.t_sl, kES);
  const char* d_c = bonus ? nullptr : row_ptr(a.d, int64_t(b) * a.d_sb + int64_t(j) * a.d_sl, kES);
  const char* d_u = bonus ? nullptr : row_ptr(a.du, int64_t(b) * a.d_sb + int64_t(j) * a.d_sl, kES);
  const float thr_t = masked ? a.thr[rt_] : -INFINITY;
  const float thr_d = (masked && !bonus) ? a.thr[rd_] : -INFINITY;
  const float omega = bonus ? 1.f : a.omega[int64_t(b) * a.om_sb + j];

  RowRegs<DT, XF, kT> rt, rd;
  float part[kT];
  auto load_pair = [&](int cc) {
    const int64_t base = int64_t(cc) * kChunk2;
    // the mass pass reads every chunk of the row exactly once: nontemporal loads
    constexpr int kA = AL ? (STAGE == kMasses ? kAlignedStream : kAligned) : kUnaligned;
    load_chunk<DT, XF, kA, kT>(rt, t_c, t_u, base, a.V, a.cfg_scale, a.inv_T, thr_t);
    if (!bonus) load_chunk<DT, XF, kA, kT>(rd, d_c, d_u, base, a.V, a.cfg_scale, a.inv_T, thr_d);
    else rd.clear();                                  // never read in mode P
  };
  if constexpr (STAGE == kMasses) load_pair(c);       // in flight before anything waits for the statistics
  ResidCoef k{rs.x, 1.f / rs.y, rs.z, bonus ? 1.f : 1.f / rs.w, omega,
              bonus ? kModeP : (a.resample_mode == 1 ? kModeVanilla : kModeOpt)};
  // Eq. g_lantern: this thread's part of the patch for chunk cc -- which of its tokens belong to the
  // rejected token's neighbour set (element j of tile t is token cc*kChunk2 + (t*256 + tid)*kE + j)
  auto lan_patch = [&](int cc) -> LanPatch {
    LanPatch lp{0u, -1, 1.f};
    if constexpr (LAN) {
      if (!bonus) {
        constexpr int kE = Vec<DT>::kE;
        const int64_t base = int64_t(cc) * kChunk2;
        auto slot = [&](int tokn) -> int {              // bit of token tokn in this thread, or -1
          const int64_t rel = int64_t(tokn) - base;
          if (rel < 0 || rel >= kChunk2) return -1;
          const int vec = int(rel) / kE;
          if ((vec & (kThreads - 1)) != (int)threadIdx.x) return -1;
          return (vec / kThreads) * kE + (int(rel) - vec * kE);
        };
        const int xd = min(max(a.tokens[int64_t(b) * a.L + j], 0), a.V - 1);
        const int m = a.lan_count[int64_t(b) * a.L + j];
        lp.agg = omega;
        lp.aggpos = slot(xd);
        const int32_t* row = a.nbr + int64_t(xd) * a.lan_k;
        int taken = 0;
        for (int jj = 0; jj < a.lan_k && taken < m; ++jj) {
          const int n = row[jj];
          if (n < 0 || n >= a.V || n == xd) continue;
          ++taken;
          const int sl = slot(n);
          if (sl >= 0) lp.zmask |= 1u << sl;
        }
      }
    }
    return lp;
  };

  if constexpr (STAGE == kMasses) {
    // only the chunk's total is needed here: per-thread sum in ascending tile order, one wave
    // reduction, one barrier (the selection launch forms its own tile totals for the chunk it picks)
    constexpr int kE = Vec<DT>::kE;
    const LanPatch lp = lan_patch(c);
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
    return;
  }

  float R, vsel;     // total mass; remaining mass to walk inside the selected chunk
  int cs = 0;        // selected chunk
  LanPatch lp_sel{0u, -1, 1.f};
  {
    // chunk masses are staged in LDS by all threads (one latency), then walked in ascending
    // order; rows with more than kStage chunks walk global memory instead
    __shared__ float cm[kStage];
    const bool staged = C <= kStage;
    // mass of chunk cc under the fallback law p, from the chunk statistics of kernel 1
    const int per = kChunk2 / a.chunk1;
    auto p_mass = [&](int cc) -> float {
      float m = 0.f;
      for (int q = cc * per; q < min((cc + 1) * per, a.c1); ++q) {
        const float2 pp = a.part[int64_t(rt_) * a.c1 + q];
        m = __fadd_rn(m, __fmul_rn(__fmul_rn(pp.y, exp2_fast(pp.x - rs.x)), k.at));
      }
      return m;
    };
    bool fallback = false;
    auto chunk_mass = [&](int cc) -> float {
      if (staged) return cm[cc];
      return fallback ? p_mass(cc) : a.chunk_R[int64_t(b) * C + cc];
    };
    if (staged) {
      for (int cc = threadIdx.x; cc < C; cc += kThreads) cm[cc] = a.chunk_R[int64_t(b) * C + cc];
      __syncthreads();
    }
    R = 0.f;
    for (int cc = 0; cc < C; ++cc) R = __fadd_rn(R, chunk_mass(cc));
    if (!(R > 0.f)) {    // no rejection possible at this position: any law is optimal, use p
      fallback = true;
      k.mode = kModeP;
      if (staged) {
        __syncthreads();
        for (int cc = threadIdx.x; cc < C; cc += kThreads) cm[cc] = p_mass(cc);
        __syncthreads();
      }
      R = 0.f;
      for (int cc = 0; cc < C; ++cc) R = __fadd_rn(R, chunk_mass(cc));
    }
    const float v = __fmul_rn(a.u_res[b], R);
    int clast = -1;
    float cbase = 0.f, cbase_last = 0.f, cum = 0.f;
    cs = -1;
    for (int cc = 0; cc < C; ++cc) {
      const float m = chunk_mass(cc);
      if (m > 0.f) {
        if (cs < 0 && __fadd_rn(cum, m) > v) { cs = cc; cbase = cum; }
        clast = cc; cbase_last = cum;
      }
      cum = __fadd_rn(cum, m);
    }
    if (cs < 0) { cs = clast; cbase = cbase_last; }
    if (cs < 0) cs = 0;
    vsel = v - cbase;
    load_pair(cs);
    lp_sel = lan_patch(cs);
    chunk_masses<DT, XF, kT, LAN>(rt, rd, k, part, sm, lp_sel);
  }
  const int off = chunk_select<DT, XF, kT, LAN>(rt, rd, k, part, vsel, sm, lp_sel);
  int token = cs * kChunk2 + max(off, 0);
  if (token >= a.V) token = a.V - 1;
  if (threadIdx.x == 0) {
    a.next_token[b] = token;
    if (a.resid_mass) a.resid_mass[b] = R;
  }
}

// ============================================================================ diagnostics
// Per-position quantities of Theorem 2 for the row pair (p_i, q_i) with relaxation omega_i:
//   alpha_i = sum_x min{q_i(x), omega_i p_i(x)} = sum_x q_i(x) f_i(x): the probability that a
//             token drawn from q_i is accepted, the factor of the expected accepted length
//             (Eq. token_exp);
//   beta_i  = sum_x [min{q_i(x), omega_i p_i(x)} - p_i(x)]_+ : half the bracket that position i
//             contributes to the total-variation bound when G* is the resampling law
//             (Theorem 2, proof Step 2); zero when omega_i <= 1.
// Both need p_i and q_i normalised, i.e. the statistics of the whole row pair first.
//   LOCAL   the row pair is one chunk (at most 16384 logits): statistics are formed here from
//           the registers, every logit is read once, results go straight to alpha / beta.
//   else    statistics come from row_stats_kernel; grid = B L x CD chunks of 8192 logits; the
//           chunk sums go to diag_part and diag_combine_kernel adds them in ascending order.
//   VER     (with LOCAL) cool_sd_verify_diagnostics: the same workgroups also leave what the
//           verify call's statistics pass leaves -- (c, S) of both rows and the logits of x~_i --
//           and B more workgroups take the bonus rows, so that the per-sequence kernel can follow
//           and no logit is read a second time for the diagnostics.
template <int DT, bool XF, int AL, int NT, bool LOCAL, bool VER = false>
__global__ __launch_bounds__(LOCAL ? 512 : kThreads) void diag_kernel(const KArgs a) {
  static_assert(LOCAL || !VER, "the fused form holds whole rows");
  constexpr int kE = Vec<DT>::kE, kES = Vec<DT>::kES;
  // the one-chunk form spreads the row pair over 512 threads so that both rows cost 64 registers
  constexpr int kTPB = LOCAL ? 512 : kThreads, kW = kTPB / 64;
  __shared__ float red[4][kW];
  const int CD = a.nchunks;
  const int pairs = a.B * a.L;
  const bool bonus_wg = VER && (int)blockIdx.x >= pairs;          // a bonus row: target only, statistics only
  const int rp = bonus_wg ? 0 : blockIdx.x / CD, c = bonus_wg ? 0 : blockIdx.x - rp * CD;   // row pair (b, i), chunk
  const int b = bonus_wg ? (int)blockIdx.x - pairs : rp / a.L, i = bonus_wg ? a.L : rp - b * a.L;
  // rows are numbered as in the verify call; the plain diagnostics call sets has_bonus = 0
  const int rt_ = b * (a.L + a.has_bonus) + i, rd_ = a.rows_t + b * a.L + (bonus_wg ? a.L - 1 : i);
  const int64_t offt = int64_t(b) * a.t_sb + int64_t(i) * a.t_sl;
  const int64_t offd = int64_t(b) * a.d_sb + int64_t(bonus_wg ? a.L - 1 : i) * a.d_sl;
  const int64_t base = int64_t(c) * (NT * kTPB * kE);
  const bool masked = XF && !LOCAL && a.top_k > 0;
  const float thr_t = masked ? a.thr[rt_] : -INFINITY;
  const float thr_d = masked ? a.thr[rd_] : -INFINITY;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;

  RowRegs<DT, XF, NT> rt, rd;
  load_chunk<DT, XF, AL, NT, kTPB, 1>(rt, row_ptr(a.t, offt, kES), row_ptr(a.tu, offt, kES), base, a.V,
                                      a.cfg_scale, a.inv_T, thr_t);
  if (!bonus_wg)
    load_chunk<DT, XF, AL, NT, kTPB, 1>(rd, row_ptr(a.d, offd, kES), row_ptr(a.du, offd, kES), base, a.V,
                                        a.cfg_scale, a.inv_T, thr_d);
  else
    rd.clear();                                         // a bonus row has no draft: zeros, results ignored
  const float omega = bonus_wg ? 1.f : a.omega[int64_t(b) * a.om_sb + i];
  // the logits of x~_i for the accept test, by one thread, requested together with the rows
  float tok_t = 0.f, tok_d = 0.f;
  if constexpr (VER) {
    if (threadIdx.x == 0 && !bonus_wg) {
      const int x = min(max(a.tokens[rp], 0), a.V - 1);
      tok_t = token_logit_any(DT, row_ptr(a.t, offt, kES), row_ptr(a.tu, offt, kES), x, XF, a.cfg_scale, a.inv_T, -INFINITY);
      tok_d = token_logit_any(DT, row_ptr(a.d, offd, kES), row_ptr(a.du, offd, kES), x, XF, a.cfg_scale, a.inv_T, -INFINITY);
    }
  }
  float sa = 0.f, sb = 0.f;
  if constexpr (LOCAL) {
    // the arithmetic is what limits this form (two exponentials per logit would), so each
    // 2^(l log2e - C) is evaluated once against the row's reference exponent and kept
    float mt = -INFINITY, md = -INFINITY;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
      for (int j = 0; j < kE; ++j) { mt = fmaxf(mt, rt.get(t, j)); md = fmaxf(md, rd.get(t, j)); }
    }
    // Each wave takes its own integer reference exponent (the ceiling of its maximum), so the
    // exponentials need not wait for a workgroup-wide maximum: changing from a wave's reference to
    // the row's is an exact power-of-two scaling, applied once per wave below.
    const float cwt = fmaxf(ceilf(wave_max(mt) * kLog2e), kRefFloor);
    const float cwd = fmaxf(ceilf(wave_max(md) * kLog2e), kRefFloor);
    float et[NT * kE], ed[NT * kE];
    float st = 0.f, sd = 0.f;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
      for (int j = 0; j < kE; ++j) {
        et[t * kE + j] = exp2_fast(__fmaf_rn(rt.get(t, j), kLog2e, -cwt));
        ed[t * kE + j] = exp2_fast(__fmaf_rn(rd.get(t, j), kLog2e, -cwd));
        st = __fadd_rn(st, et[t * kE + j]);
        sd = __fadd_rn(sd, ed[t * kE + j]);
      }
    }
    st = wave_sum(st);
    sd = wave_sum(sd);
    if (lane == 0) { red[0][wv] = cwt; red[1][wv] = cwd; red[2][wv] = st; red[3][wv] = sd; }
    __syncthreads();
    float Ct = red[0][0], Cd = red[1][0];
#pragma unroll
    for (int w = 1; w < kW; ++w) { Ct = fmaxf(Ct, red[0][w]); Cd = fmaxf(Cd, red[1][w]); }
    float St = 0.f, Sd = 0.f;
#pragma unroll
    for (int w = 0; w < kW; ++w) {
      St = __fadd_rn(St, red[2][w] * exp2_fast(red[0][w] - Ct));
      Sd = __fadd_rn(Sd, red[3][w] * exp2_fast(red[1][w] - Cd));
    }
    if constexpr (VER) {
      if (threadIdx.x == 0) {
        a.part[int64_t(rt_) * a.c1] = make_float2(Ct, St);
        if (!bonus_wg) {
          a.part[int64_t(rd_) * a.c1] = make_float2(Cd, Sd);
          a.tok_logit[rt_] = tok_t;
          a.tok_logit[rd_] = tok_d;
        }
      }
      if (bonus_wg) return;
    }
    // 1/S and this wave's change of reference in one factor
    const float at = __fmul_rn(exp2_fast(cwt - Ct), 1.f / St), ad = __fmul_rn(exp2_fast(cwd - Cd), 1.f / Sd);
#pragma unroll
    for (int n = 0; n < NT * kE; ++n) {
      const float p = __fmul_rn(et[n], at), q = __fmul_rn(ed[n], ad);
      const float m = fminf(q, __fmul_rn(omega, p));
      sa = __fadd_rn(sa, m);
      sb = __fadd_rn(sb, fmaxf(__fsub_rn(m, p), 0.f));
    }
    __syncthreads();                                              // red is reused below
  } else {
    float Ct, St, Cd, Sd;
    combine_row(a, rt_, Ct, St);
    combine_row(a, rd_, Cd, Sd);
    const float at = 1.f / St, ad = 1.f / Sd;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
      for (int j = 0; j < kE; ++j) {
        const float p = __fmul_rn(exp2_fast(__fmaf_rn(rt.get(t, j), kLog2e, -Ct)), at);
        const float q = __fmul_rn(exp2_fast(__fmaf_rn(rd.get(t, j), kLog2e, -Cd)), ad);
        const float m = fminf(q, __fmul_rn(omega, p));
        sa = __fadd_rn(sa, m);
        sb = __fadd_rn(sb, fmaxf(__fsub_rn(m, p), 0.f));
      }
    }
  }
  sa = wave_sum(sa);
  sb = wave_sum(sb);
  if (lane == 0) { red[0][wv] = sa; red[1][wv] = sb; }
  __syncthreads();
  if (threadIdx.x == 0) {
    float A = 0.f, Bv = 0.f;
#pragma unroll
    for (int w = 0; w < kW; ++w) { A = __fadd_rn(A, red[0][w]); Bv = __fadd_rn(Bv, red[1][w]); }
    if constexpr (LOCAL) {
      a.alpha[rp] = A;
      a.beta[rp] = Bv;
    } else {
      a.diag_part[int64_t(rp) * CD + c] = make_float2(A, Bv);
    }
  }
}

// Adds the chunk sums of every row pair in ascending chunk order: one thread per row pair.
__global__ __launch_bounds__(kThreads) void diag_combine_kernel(const KArgs a) {
  const int rp = blockIdx.x * kThreads + threadIdx.x;
  if (rp >= a.B * a.L) return;
  const float2* p = a.diag_part + int64_t(rp) * a.nchunks;
  float A = 0.f, Bv = 0.f;
  for (int c = 0; c < a.nchunks; ++c) {
    const float2 v = p[c];
    A = __fadd_rn(A, v.x);
    Bv = __fadd_rn(Bv, v.y);
  }
  a.alpha[rp] = A;
  a.beta[rp] = Bv;
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
      } else {                           // 16384 < V <= 65536: 1024 threads, statistics per 8192 logits
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
    if (a.resample_only && a.top_k > 0 && a.d == nullptr && a.V <= kChunk && !a.stats_only) {
      // the drafting stage's draw under truncation: one launch
      constexpr int kA = AL ? kAligned : kUnaligned;
      if (ev) (void)hipEventRecord(ev[1], stream);
      if (a.tu != nullptr) hipLaunchKernelGGL((resample_topk_kernel<DT, kA, 1>), dim3((unsigned)a.B), dim3(kThreadsK), 0, stream, a);
      else hipLaunchKernelGGL((resample_topk_kernel<DT, kA, 0>), dim3((unsigned)a.B), dim3(kThreadsK), 0, stream, a);
      hipError_t er = checked("resample_topk_kernel");
      if (ev) (void)hipEventRecord(ev[2], stream);
      return er;
    }
  }
  if (a.resample_only && a.top_k == 0 && a.V <= kChunk && !a.stats_only) {   // short rows: one launch
    if (ev) (void)hipEventRecord(ev[1], stream);
    hipLaunchKernelGGL((resample_whole_kernel<DT, XF, AL>), dim3((unsigned)a.B), dim3(kThreadsW), 0, stream, a);
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

template <int DT, bool XF, bool AL>
static hipError_t launch_rest(const KArgs& a, hipStream_t stream) {
  constexpr int kT = Vec<DT>::kT;
  hipError_t e;
  if (a.cs != a.c1 && !a.accept_combines) {   // rows have many statistics chunks: pre-combine them, one wave per row
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
  if (!a.resample_only) {     // several chunks: find tau once per sequence
    hipLaunchKernelGGL((accept_kernel<DT, XF>), dim3(gB), dim3(kThreadsW), 0, stream, a);
    e = checked("accept_kernel");
    if (e != hipSuccess) return e;
  }
  const int64_t grid2 = int64_t(a.B) * a.nchunks;
  if (a.lan_resample)
    hipLaunchKernelGGL((sequence_kernel<DT, XF, AL, kT / 2, kMasses, true>), dim3((unsigned)grid2), dim3(kThreads), 0, stream, a);
  else
    hipLaunchKernelGGL((sequence_kernel<DT, XF, AL, kT / 2, kMasses, false>), dim3((unsigned)grid2), dim3(kThreads), 0, stream, a);
  e = checked("sequence_kernel (masses)");
  if (e != hipSuccess) return e;
  if (a.lan_resample)
    hipLaunchKernelGGL((sequence_kernel<DT, XF, AL, kT / 2, kSelect, true>), dim3(gB), dim3(kThreads), 0, stream, a);
  else
    hipLaunchKernelGGL((sequence_kernel<DT, XF, AL, kT / 2, kSelect, false>), dim3(gB), dim3(kThreads), 0, stream, a);
  return checked("sequence_kernel");
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
static hipError_t launch_diag_typed(const KArgs& a, bool local, hipStream_t stream) {
  constexpr int kT = Vec<DT>::kT;
  constexpr int kA = AL ? kAligned : kUnaligned;
  (void)hipGetLastError();
  const int64_t pairs = int64_t(a.B) * a.L;
  if (local) {
    hipLaunchKernelGGL((diag_kernel<DT, XF, kA, kT / 2, true>), dim3((unsigned)pairs), dim3(512), 0, stream, a);
    return checked("diag_kernel (one chunk)");
  }
  hipError_t e = launch_stats_any<DT, XF, AL>(a, stream);
  if (e != hipSuccess) return e;
  if (a.cs != a.c1) {
    const int64_t gridc = (int64_t(a.rows_t) + a.rows_d + kWaves - 1) / kWaves;
    hipLaunchKernelGGL(combine_rows_kernel, dim3((unsigned)gridc), dim3(kThreads), 0, stream, a);
    e = checked("combine_rows_kernel");
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL((diag_kernel<DT, XF, kA, kT / 2, false>), dim3((unsigned)(pairs * a.nchunks)), dim3(kThreads), 0,
                     stream, a);
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

hipError_t launch_diagnostics(const KArgs& a, int dtype, bool xf, bool local, hipStream_t stream) {
  if (dtype == kDtBF16) {
    if (xf) return a.aligned ? launch_diag_typed<kDtBF16, true, true>(a, local, stream)
                             : launch_diag_typed<kDtBF16, true, false>(a, local, stream);
    return a.aligned ? launch_diag_typed<kDtBF16, false, true>(a, local, stream)
                     : launch_diag_typed<kDtBF16, false, false>(a, local, stream);
  }
  if (xf) return a.aligned ? launch_diag_typed<kDtF32, true, true>(a, local, stream)
                           : launch_diag_typed<kDtF32, true, false>(a, local, stream);
  return a.aligned ? launch_diag_typed<kDtF32, false, true>(a, local, stream)
                   : launch_diag_typed<kDtF32, false, false>(a, local, stream);
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
