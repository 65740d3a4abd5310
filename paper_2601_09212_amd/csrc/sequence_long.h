// Second step of a verify call on rows longer than 16384 logits (chunk masses, then selection).
// Part of the one translation unit verify_kernels.hip (included there, inside namespace csd,
// after device_utils.h, kernels.h and topk.h); not a stand-alone header.
#pragma once

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
