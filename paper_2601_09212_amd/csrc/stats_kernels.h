// Statistics pass (the HBM-bound launch of a verify call): row_stats_kernel and the neighbour
// aggregation that rides along in its launch.
#pragma once
#include "kernel_common.h"
#include "topk.h"

namespace csd {

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
    // grid.y counts the target rows of the window of positions, then its draft rows (the window
    // is the whole sequence unless the call verifies in rounds)
    const int wt = (a.win_hi ? min(a.win_hi, per_t) : per_t) - a.win_lo;
    o.b = blockIdx.z;
    o.is_draft = (int)blockIdx.y >= wt;
    o.i = a.win_lo + (o.is_draft ? blockIdx.y - wt : blockIdx.y);
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
// The value is clamped into [0, V-1] wherever it is used as an address, like in every other kernel.
__device__ __forceinline__ int load_draft_token(const KArgs& a, const RowRef& rw) {
  if (a.tokens == nullptr || rw.i >= a.L) return -1;
  int z = 0;
  asm volatile("" : "+v"(z));
  return min(max(a.tokens[int64_t(rw.b) * a.L + rw.i + z], 0), a.V - 1);
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
  // The set is an integer decision (which neighbours belong): it is taken in fp64 -- weights from
  // the exact logit differences, running sum in list order -- so that it agrees with exact
  // arithmetic wherever the inequality is not a tie to fifteen digits.  One wave, k values: free.
  double cum = 0.0;
  const double lam = (double)a.lan_lambda;
  int m = 0;
  if (lx > -INFINITY) {                       // p(x~) = 0 admits no neighbour: nothing is below 0
    for (int j0 = 0; j0 < a.lan_k; j0 += 64) {
      const int j = j0 + lane;
      const int n = j < a.lan_k ? row[j] : -1;
      const bool valid = n >= 0 && n < a.V && n != x;
      const float ln = valid ? token_logit_any(dt, cond, uncond, n, xf, a.cfg_scale, a.inv_T, thr) : -INFINITY;
      const double w = valid ? exp2_d(((double)ln - (double)lx) * kLog2eD) : 0.0;
      double incl = w;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const double t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
      }
      incl += cum;
      const unsigned long long bv = __ballot(valid);
      const unsigned long long bf = __ballot(valid && !(incl < lam));
      if (bf) {                                // the first neighbour that does not fit ends the set
        const int fl = __ffsll((long long)bf) - 1;
        m += __popcll(bv & ((1ull << fl) - 1ull));
        // the running sum before lane fl: weights of skipped lanes are zero, so it is the sum
        // over the members taken so far
        if (fl > 0) cum = __shfl(incl, fl - 1, 64);
        break;
      }
      m += __popcll(bv);
      cum = __shfl(incl, 63, 64);
    }
  }
  if (lane == 0) {
    a.lan_omega[pos] = (float)(1.0 + cum);
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
  if constexpr (G3) {
    // verification in rounds: a sequence that has its rejection needs no further row
    if (a.win_lo > 0 && a.tau_ws[rw.b] >= 0) return;
  }
  const int r = rw.r;
  const int64_t base = int64_t(c) * (NT * kThreads * kE);
  // the first workgroup of every sequence clears the sequence's ticket for the long-row tail launch
  // that follows in the stream
  if (c == 0 && rw.i == 0 && !rw.is_draft && threadIdx.x == 0) a.ticket[rw.b] = 0;

  // rows longer than one workgroup under top-k: the threshold was selected by the radix passes
  float thr = -INFINITY;
  if constexpr (XF) {
    if (a.top_k > 0) thr = a.thr[r];
  }
  RowRegs<DT, XF, NT> x;
  load_chunk<DT, XF, AL, NT>(x, rw.cond, rw.uncond, base, a.V, a.cfg_scale, a.inv_T, thr);
  const int tok = load_draft_token(a, rw);     // after the chunk's loads in program order, used after them
  // the (transformed) logit of x~_i for the accept test of the next kernel, taken from the
  // registers of the thread that holds it: element e of vector (tile k, thread t) is token
  // base + (k*256 + t)*kE + e
  if (tok >= 0) {
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

}  // namespace csd
