// Top-k truncation: whole-row statistics with threshold selection (row_stats_topk_kernel), the
// draft-side draw in one launch (resample_topk_kernel) and the radix passes for rows beyond
// 65536 logits.
#pragma once
#include "exact_draw.h"
#include "stats_kernels.h"

namespace csd {

// Statistics of whole rows under top-k truncation: one workgroup of TPB threads per row,
// ROW / TPB transformed logits per thread in registers (ROW = 16384 with 512 threads; 32768 or
// 65536 with 1024 threads for vocabularies up to 32K / 64K).  The k-th largest value of the row is selected
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
  if (rw.i == 0 && !rw.is_draft && threadIdx.x == 0) a.ticket[rw.b] = 0;   // for the long-row tail launch that follows
  topk_prepare(ts);                                     // the barrier inside topk_threshold orders it
  RowRegs<DT, true, kVW> x;
  // vector k of thread t is vector k*TPB + t of the row; a row that fills the workgroup's span
  // exactly needs no range test on its vectors
  if (AL != kUnaligned && a.V == ROW)
    load_chunk<DT, true, kAlignedFull, kVW, TPB, 1, 4, GD>(x, rw.cond, rw.uncond, 0, a.V, a.cfg_scale, a.inv_T, -INFINITY);
  else
    load_chunk<DT, true, AL, kVW, TPB, 1, 4, GD>(x, rw.cond, rw.uncond, 0, a.V, a.cfg_scale, a.inv_T, -INFINITY);
  // the raw logits of x~_i, requested now and used at the very end
  const int tok = load_draft_token(a, rw);
  float tok_c = 0.f, tok_u = 0.f;
  if (tok >= 0 && threadIdx.x == 0) {
    tok_c = load_elem<DT>(rw.cond, tok);
    if (rw.uncond) tok_u = load_elem<DT>(rw.uncond, tok);
  }
  float row_max;
  const TopkBracket br = topk_bracket<kVW * kE, TPB>(x.w, a.top_k, ts, row_max);
  const float c = fmaxf(ceilf(row_max * kLog2e), kRefFloor);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  float thr;
  if (kSub == 1 && !br.exact) {
    // One pass does both jobs: values above the bracket are kept whatever the threshold turns
    // out to be, so their weights are summed while the few candidates are still being collected;
    // the candidates at or above the threshold are added once they are ranked.
    float s = 0.f;
#pragma unroll
    for (int n = 0; n < kVW * kE; ++n) {
      const float l = __uint_as_float(x.w[n]);
      const float e = exp2_fast(__fmaf_rn(l, kLog2e, -c));
      const bool above = l > br.g_hi;
      s += above ? e : 0.f;
      if (!above && l >= br.g_lo) {
        const int bk = bucket_of(l, br.hi, br.scale);
        if (bk == br.bsel) ts.list[atomicAdd(&ts.n_list, 1u)] = l;
        else if (bk < br.bsel) s += e;
      }
    }
    s = wave_sum(s);
    if (lane == 0) red_s[0][wv] = s;
    __syncthreads();
    // Rank the candidates.  A candidate with fewer than kk larger ones is kept; kept candidates
    // leave their weights in rank order (equal values in any order: their weights are equal), so
    // that the sum below does not depend on the order in which the list was filled.
    float* kept = reinterpret_cast<float*>(ts.hist);     // the histogram is no longer needed
    for (uint32_t i = threadIdx.x; i < br.nb; i += TPB) {
      const float v = ts.list[i];
      uint32_t g = 0, ge = 0, eq_before = 0;
      for (uint32_t j = 0; j < br.nb; ++j) {
        const float w = ts.list[j];
        g += w > v;
        ge += w >= v;
        eq_before += (j < i) && (w == v);
      }
      if (g < br.kk) {
        kept[g + eq_before] = exp2_fast(__fmaf_rn(v, kLog2e, -c));
        if (br.kk <= ge) { ts.thr = v; ts.n_keep = ge; }
      }
    }
    __syncthreads();
    thr = ts.thr;
    if (wv == 0) {
      float cs = 0.f;
      for (uint32_t j = lane; j < ts.n_keep; j += 64) cs += kept[j];
      cs = wave_sum(cs);
      if (lane == 0 && a.c1 > 0) {
        float S = red_s[0][0];
#pragma unroll
        for (int w = 1; w < kW; ++w) S = __fadd_rn(S, red_s[0][w]);
        a.part[int64_t(r) * a.c1] = make_float2(c, __fadd_rn(S, cs));
      }
    }
  } else {
    thr = kth_from_bracket<kVW * kE, TPB>(x.w, br, ts);
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
// (TPB, ROW) = (512, 16384), or 1024 threads for rows of up to 32768 / 65536 logits, as in
// row_stats_topk_kernel.
template <int DT, int AL, int GD, int TPB = kThreadsK, int ROW = kChunk>
__global__ __launch_bounds__(TPB) void resample_topk_kernel(const KArgs a) {
  constexpr int kE = Vec<DT>::kE, kES = Vec<DT>::kES;
  constexpr int kVW = ROW / (TPB * kE);                // tiles: 4 (bf16) / 8 (fp32) on rows of 16384 logits
  constexpr int kW = TPB / 64;
  static_assert(kVW <= 8, "tile_part holds up to 8 tiles");
  __shared__ TopkSmem<TPB> ts;
  __shared__ float tile_part[kW][8];
  __shared__ float scan_tot[kW];
  __shared__ int pick_first[kW], pick_last[kW];
  __shared__ int needs64;
  __shared__ ExactSmem<TPB> smx;
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
  const bool tile_fallback = ks < 0;
  if (tile_fallback) { ks = klast; base = base_last; }
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
  if (tid == 0) needs64 = 0;
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
  const bool thread_fallback = win == 0x7fffffff;
  if (thread_fallback) win = last_pos;
  // level 3: element, by the winning thread
  int token = 0;
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
    const bool element_fallback = found < 0;
    if (element_fallback) found = last;
    token = min((ks * TPB + win) * kE + found, a.V - 1);
    // the law is p itself (mass 1): fp32 resolves it unless a level's roundings disagreed
    if (tile_fallback || thread_fallback || element_fallback) needs64 = 1;
  }
  __syncthreads();
  float mass = 1.f;                                      // the law is p itself
  if (needs64 || a.exact_draw) {
    const ExactJob job{{row_ptr(a.t, int64_t(b) * a.t_sb, kES), row_ptr(a.tu, int64_t(b) * a.t_sb, kES), thr, (double)c},
                       {nullptr, nullptr, -INFINITY, 0.0}, DT, true, a.V, a.cfg_scale, a.inv_T, 1.f, kModeP, nullptr, 0, 0, 0};
    token = exact_draw<TPB>(job, u, mass, smx);
    win = 0;
  }
  if (tid == win) {
    a.next_token[b] = token;
    if (a.resid_mass) a.resid_mass[b] = mass;
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

}  // namespace csd
