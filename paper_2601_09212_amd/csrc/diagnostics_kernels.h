// Per-position terms of Theorem 2 (alpha_i, beta_i).
#pragma once
#include "sequence_common.h"
#include "stats_kernels.h"

namespace csd {

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

}  // namespace csd
