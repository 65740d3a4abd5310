// Host side of the C ABI shared by the product library (api.hip) and the benchmark library
// (bench_api.hip): argument validation, workspace layout, and the translation of a call into the
// kernel arguments.  Everything here is a pure function of its arguments: no file-scope state.
#pragma once
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <algorithm>

#include "cool_sd.h"
#include "device_utils.h"
#include "kernels.h"

namespace csd_api {
namespace {


constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layout {
  size_t seq_stat, ticket, chunk_R, thr, tok_logit, rowstat, part, diag_part, lan, rk_hist, rk_state, total;
};

// cool_sd_verify_lantern only
struct LanternArgs {
  const int32_t* nbr;
  int32_t k;
  float lambda;
  float* p_agg;
  int32_t* count;
};

// rows: all logit rows (target + draft); c1: statistics chunks per row; C: sampling chunks per row.
// pairs x CD: (alpha, beta) chunk sums of the diagnostics call (0 pairs: region absent).
// lan_pairs: B L of a call with neighbour aggregation (its omega and member counts), else 0.
// rk_rows: rows of a call that selects top-k thresholds by radix passes (long rows), else 0.
Layout make_layout(int64_t B, int64_t rows, int64_t c1, int64_t C, int64_t pairs = 0, int64_t CD = 0,
                   int64_t lan_pairs = 0, int64_t rk_rows = 0) {
  Layout o{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t at = off; off = align_up(off + bytes); return at; };
  o.seq_stat = take(size_t(B) * 16);
  o.ticket = take(size_t(B) * 8);       // tickets, then the state of a verification in rounds
  o.chunk_R = take(size_t(B) * C * 4);
  o.thr = take(size_t(rows) * 4);
  o.tok_logit = take(size_t(rows) * 4);
  o.rowstat = take(size_t(rows) * 8);
  o.part = take(size_t(rows) * c1 * 8);
  o.diag_part = take(size_t(pairs) * CD * 8);
  o.lan = take(size_t(lan_pairs) * 8);
  o.rk_hist = take(size_t(rk_rows) * 2048 * 4);
  o.rk_state = take(size_t(rk_rows) * 8);
  o.total = off;
  return o;
}

// Statistics-kernel chunking: tiles per chunk (of Vec::kT, kT/2, kT/4 = 16384, 8192, 4096
// logits).  Small chunks keep more workgroups in flight; top-k needs the whole row in one.
struct Chunking { int nt1, chunk1; int64_t c1; int nt2; int64_t c2; };
Chunking pick_chunking(const cool_sd_params* p, int64_t rows) {
  const int kT = (p->dtype == COOL_SD_BF16) ? 8 : 16;
  const int kE = (p->dtype == COOL_SD_BF16) ? 8 : 4;
  const bool one_chunk = p->V <= csd::kChunk;     // the sampled row fits one workgroup's registers
  int nt = kT / 2;
  if (p->top_k > 0 && one_chunk) nt = kT;      // the top-k kernel holds a whole row
  else if (one_chunk && rows * ((p->V + 8191) / 8192) < 2048) nt = kT / 4;
  Chunking c;
  c.nt1 = nt;
  c.chunk1 = nt * 256 * kE;
  c.c1 = (int64_t(p->V) + c.chunk1 - 1) / c.chunk1;
  // sampling kernel: one 16384-logit chunk, or 8192-logit chunks (then equal to the statistics chunks)
  c.nt2 = one_chunk ? kT : kT / 2;
  const int64_t chunk2 = int64_t(c.nt2) * 256 * kE;
  c.c2 = (int64_t(p->V) + chunk2 - 1) / chunk2;
  return c;
}


bool params_ok(const cool_sd_params* p, bool for_resample, bool lantern = false) {
  if (!p) return false;
  if (p->B < 1 || p->V < 1) return false;
  if (!for_resample && (p->L < 1 || p->L > 4096)) return false;
  if (p->dtype != COOL_SD_F32 && p->dtype != COOL_SD_BF16) return false;
  if (p->t_stride_b < 0 || p->d_stride_b < 0) return false;
  if (!for_resample && (p->t_stride_l < 0 || p->d_stride_l < 0 || p->omega_stride_b < 0)) return false;
  if (!for_resample && p->has_bonus != 0 && p->has_bonus != 1) return false;
  if (p->top_k < 0 || p->top_k > p->V) return false;
  if (!(p->temperature > 0.f) || !isfinite(p->temperature)) return false;
  if (!isfinite(p->cfg_scale)) return false;
  if (p->resample_mode != COOL_SD_RESAMPLE_OPT && p->resample_mode != COOL_SD_RESAMPLE_VANILLA &&
      !(lantern && p->resample_mode == COOL_SD_RESAMPLE_LANTERN))
    return false;
  if ((p->flags & ~(COOL_SD_FLAG_EARLY_EXIT | COOL_SD_FLAG_CHECK_TOKENS | COOL_SD_FLAG_EXACT_DRAW)) != 0) return false;
  const int64_t L = for_resample ? 1 : p->L;
  const int64_t rows = for_resample ? p->B : int64_t(p->B) * (L + p->has_bonus);
  if (2 * rows * ((int64_t(p->V) + 4095) / 4096) > 0x7fffffffLL) return false;   // grid size
  return true;
}

// Option bits of a call.  A library built with COOL_SD_CHECKED_BUILD (libcool_sd_checked.so, the
// debug build) turns the draft-token check on for every verify call.
inline int call_flags(const cool_sd_params* p) {
#ifdef COOL_SD_CHECKED_BUILD
  return p->flags | COOL_SD_FLAG_CHECK_TOKENS;
#else
  return p->flags;
#endif
}

// How a verify call with these parameters honours COOL_SD_FLAG_EARLY_EXIT (cool_sd_early_exit_form).
// aligned: every row starts on a 16-byte boundary and V is a multiple of a 16-byte vector.
inline int early_exit_form(const cool_sd_params* p, bool aligned) {
  if (!(p->flags & COOL_SD_FLAG_EARLY_EXIT) || p->top_k != 0) return COOL_SD_EARLY_EXIT_NONE;
  if (p->V <= csd::kChunk) return (aligned && p->L <= 1024) ? COOL_SD_EARLY_EXIT_SEQUENCE : COOL_SD_EARLY_EXIT_NONE;
  // rounds: a row's chunk statistics fit one wave, and the three-dimensional grid holds the call
  const Chunking ch = pick_chunking(p, int64_t(p->B) * (2 * int64_t(p->L) + p->has_bonus));
  return (ch.c1 <= 64 && p->B <= 65535) ? COOL_SD_EARLY_EXIT_ROUNDS : COOL_SD_EARLY_EXIT_NONE;
}

inline bool is_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Workspace layout of one verify / stand-alone resample call, with the chunking it runs with.
// has_draft: a draft tensor is given; lan: neighbour aggregation; with_diag: the diagnostics pass
// follows on the statistics this call leaves (8192-logit chunks).
struct CallPlan { Chunking ch; Layout lay; int64_t L, rows_t, rows_d, C, CD; int hb; bool radix; };
CallPlan plan_call(const cool_sd_params* p, bool resample_only, bool has_draft, bool lan, bool with_diag) {
  CallPlan o;
  o.L = resample_only ? 1 : p->L;
  o.hb = resample_only ? 0 : p->has_bonus;
  o.rows_t = resample_only ? p->B : int64_t(p->B) * (o.L + o.hb);
  o.rows_d = has_draft ? int64_t(p->B) * o.L : 0;
  o.ch = pick_chunking(p, o.rows_t + o.rows_d);
  o.C = o.ch.c2;
  o.radix = p->top_k > 0 && p->V > 4 * csd::kChunk;
  const int64_t pairs = with_diag ? int64_t(p->B) * o.L : 0;
  o.CD = with_diag ? (int64_t(p->V) + 8191) / 8192 : 0;
  o.lay = make_layout(p->B, o.rows_t + o.rows_d, o.ch.c1, o.C, pairs, o.CD, lan ? int64_t(p->B) * o.L : 0,
                      o.radix ? o.rows_t + o.rows_d : 0);
  return o;
}

int run(const cool_sd_params* p, bool resample_only,
        const void* t, const void* tu, const void* d, const void* du,
        const int32_t* tokens, const float* omega, const float* u_acc, const float* u_res,
        int32_t* accept_len, int32_t* next_token, float* p_tok, float* q_tok, float* f,
        float* resid_mass, void* ws, size_t ws_bytes, void* stream, const LanternArgs* lan = nullptr,
        float* alpha = nullptr, float* beta = nullptr, bool stats_only = false) {
  const CallPlan pl = plan_call(p, resample_only, d != nullptr, lan != nullptr, alpha != nullptr);
  const int64_t L = pl.L, rows_t = pl.rows_t, rows_d = pl.rows_d, C = pl.C, CD = pl.CD;
  const int hb = pl.hb;
  const Chunking& ch = pl.ch;
  const Layout& lay = pl.lay;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0 || ws_bytes < lay.total) return COOL_SD_EWORKSPACE;

  const int kE = (p->dtype == COOL_SD_BF16) ? 8 : 4;
  bool aligned = (p->V % kE == 0) && is_aligned16(t) && (p->t_stride_b % kE == 0);
  if (!resample_only) aligned = aligned && (p->t_stride_l % kE == 0);
  if (tu) aligned = aligned && is_aligned16(tu);
  if (d) {
    aligned = aligned && is_aligned16(d) && (p->d_stride_b % kE == 0);
    if (!resample_only) aligned = aligned && (p->d_stride_l % kE == 0);
  }
  if (du) aligned = aligned && is_aligned16(du);

  char* w = static_cast<char*>(ws);
  csd::KArgs a{};
  a.t = t; a.tu = tu; a.d = d; a.du = du;
  a.tokens = tokens; a.omega = omega; a.u_acc = u_acc; a.u_res = u_res;
  a.accept_len = accept_len; a.next_token = next_token;
  a.p_tok = p_tok; a.q_tok = q_tok; a.f = f; a.resid_mass = resid_mass;
  a.t_sb = p->t_stride_b; a.d_sb = p->d_stride_b;
  a.t_sl = resample_only ? 0 : p->t_stride_l;
  a.d_sl = resample_only ? 0 : p->d_stride_l;
  a.om_sb = resample_only ? 1 : p->omega_stride_b;
  a.B = p->B; a.L = (int32_t)L; a.V = p->V; a.has_bonus = hb;
  a.top_k = p->top_k; a.resample_mode = p->resample_mode;
  a.resample_only = resample_only ? 1 : 0;
  a.aligned = aligned ? 1 : 0;
  a.stats_only = stats_only ? 1 : 0;
  a.exact_draw = (p->flags & COOL_SD_FLAG_EXACT_DRAW) ? 1 : 0;
  const int form = (resample_only || lan || alpha || stats_only) ? COOL_SD_EARLY_EXIT_NONE : early_exit_form(p, aligned);
  a.early_exit = form == COOL_SD_EARLY_EXIT_SEQUENCE ? 1 : 0;
  a.windowed = form == COOL_SD_EARLY_EXIT_ROUNDS ? 1 : 0;
  if (lan) {
    // Eq. f_lantern is Eq. relax with a data-dependent omega_i >= 1 that lantern_agg_kernel leaves
    // in the workspace; with f >= f^van the optimal law G* is [p - q]_+ (Proposition on the design
    // of G), so OPT runs the vanilla residual
    a.nbr = lan->nbr; a.lan_k = lan->k; a.lan_lambda = lan->lambda;
    a.lan_omega = reinterpret_cast<float*>(w + lay.lan);
    a.lan_count = reinterpret_cast<int32_t*>(w + lay.lan + size_t(p->B) * L * 4);
    a.p_agg_out = lan->p_agg; a.count_out = lan->count;
    a.lan_resample = p->resample_mode == COOL_SD_RESAMPLE_LANTERN ? 1 : 0;
    a.omega = a.lan_omega;
    a.om_sb = L;
    a.resample_mode = COOL_SD_RESAMPLE_VANILLA;
  }
  // beyond ~128 MB the logits cannot stay in L2 / Infinity Cache until the sequence kernel re-reads a row
  a.stream_loads = (double(rows_t + rows_d) * p->V * (p->dtype == COOL_SD_BF16 ? 2 : 4) * (tu ? 2 : 1)) > 128e6 ? 1 : 0;
  a.nchunks = (int32_t)C; a.nt2 = ch.nt2;
  // long-row tail launch: about 1024 workgroups in all (four per compute unit: enough loads in
  // flight to saturate HBM without queueing them so deep that the launch's few dependent loads
  // wait behind them), at most one per chunk, at least one per eight chunks
#ifndef CSD_TAIL_TARGET
#define CSD_TAIL_TARGET 1024
#endif
  a.tail_groups = (int32_t)std::max<int64_t>((C + 7) / 8, std::min<int64_t>(C, CSD_TAIL_TARGET / p->B));
  a.cfg_scale = p->cfg_scale;
  a.inv_T = 1.0f / p->temperature;
  a.rows_t = (int32_t)rows_t; a.rows_d = (int32_t)rows_d;
  a.nt1 = ch.nt1; a.chunk1 = ch.chunk1; a.c1 = (int32_t)ch.c1;
  a.chunk_R = reinterpret_cast<float*>(w + lay.chunk_R);
  a.seq_stat = reinterpret_cast<float4*>(w + lay.seq_stat);
  a.ticket = reinterpret_cast<int32_t*>(w + lay.ticket);
  a.tau_ws = a.ticket + p->B;
  a.thr = reinterpret_cast<float*>(w + lay.thr);
  a.tok_logit = reinterpret_cast<float*>(w + lay.tok_logit);
  a.part = reinterpret_cast<float2*>(w + lay.part);
  a.rowstat = reinterpret_cast<float2*>(w + lay.rowstat);
  a.rk_hist = reinterpret_cast<uint32_t*>(w + lay.rk_hist);
  a.rk_state = reinterpret_cast<uint32_t*>(w + lay.rk_state);
  const bool direct = ch.c1 <= 4;
  a.stat = direct ? a.part : a.rowstat;
  a.cs = direct ? (int32_t)ch.c1 : 1;
  // with many chunks per row the verify path folds their combination into accept_kernel; the
  // stand-alone resample has no such kernel, and the neighbour aggregation reads row statistics
  // before it
  a.accept_combines = (!direct && !resample_only && !lan) ? 1 : 0;

  const bool xf = (tu != nullptr) || (p->temperature != 1.0f) || (p->top_k > 0);
  hipError_t e = csd::launch_verify(a, p->dtype, xf, static_cast<hipStream_t>(stream));
  if (e == hipSuccess && !stats_only && !resample_only && (call_flags(p) & COOL_SD_FLAG_CHECK_TOKENS))
    e = csd::launch_check_tokens(a, static_cast<hipStream_t>(stream));
  if (e == hipSuccess && alpha && !stats_only) {
    // Theorem 2's per-position terms from the statistics (and thresholds) the verify call has just
    // left in the workspace: the logits are read once more, not twice
    a.alpha = alpha; a.beta = beta;
    a.diag_part = reinterpret_cast<float2*>(w + lay.diag_part);
    a.nchunks = (int32_t)CD;
    e = csd::launch_diagnostics(a, p->dtype, xf, /*local=*/false, static_cast<hipStream_t>(stream), /*have_stats=*/true);
  }
  return e == hipSuccess ? COOL_SD_OK : COOL_SD_ELAUNCH;
}

// cool_sd_diagnostics: alpha_i, beta_i of every (target, draft) row pair.  The bonus row, if the
// target tensor has one, is skipped through the strides.
int run_diag(const cool_sd_params* p, const void* t, const void* tu, const void* d, const void* du,
             const float* omega, float* alpha, float* beta, void* ws, size_t ws_bytes, void* stream) {
  const int64_t pairs = int64_t(p->B) * p->L;
  const Chunking ch = pick_chunking(p, 2 * pairs);
  const bool local = p->top_k == 0 && p->V <= csd::kChunk;
  const int64_t CD = local ? 1 : (int64_t(p->V) + 8191) / 8192;
  const bool radix = p->top_k > 0 && p->V > 4 * csd::kChunk;
  const Layout lay = make_layout(p->B, 2 * pairs, ch.c1, 1, pairs, CD, 0, radix ? 2 * pairs : 0);
  if (!ws || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0 || ws_bytes < lay.total) return COOL_SD_EWORKSPACE;

  const int kE = (p->dtype == COOL_SD_BF16) ? 8 : 4;
  bool aligned = (p->V % kE == 0) && is_aligned16(t) && is_aligned16(d) && (p->t_stride_b % kE == 0) &&
                 (p->t_stride_l % kE == 0) && (p->d_stride_b % kE == 0) && (p->d_stride_l % kE == 0);
  if (tu) aligned = aligned && is_aligned16(tu) && is_aligned16(du);

  char* w = static_cast<char*>(ws);
  csd::KArgs a{};
  a.t = t; a.tu = tu; a.d = d; a.du = du;
  a.omega = omega; a.alpha = alpha; a.beta = beta;
  a.t_sb = p->t_stride_b; a.t_sl = p->t_stride_l; a.d_sb = p->d_stride_b; a.d_sl = p->d_stride_l;
  a.om_sb = p->omega_stride_b;
  a.B = p->B; a.L = p->L; a.V = p->V; a.has_bonus = 0;
  a.top_k = p->top_k; a.resample_mode = p->resample_mode;
  a.aligned = aligned ? 1 : 0;
  a.stream_loads = 0;     // every row is read again by the second pass
  a.nchunks = (int32_t)CD;
  a.cfg_scale = p->cfg_scale;
  a.inv_T = 1.0f / p->temperature;
  a.rows_t = (int32_t)pairs; a.rows_d = (int32_t)pairs;
  a.nt1 = ch.nt1; a.chunk1 = ch.chunk1; a.c1 = (int32_t)ch.c1;
  a.ticket = reinterpret_cast<int32_t*>(w + lay.ticket);
  a.thr = reinterpret_cast<float*>(w + lay.thr);
  a.tok_logit = reinterpret_cast<float*>(w + lay.tok_logit);
  a.part = reinterpret_cast<float2*>(w + lay.part);
  a.rowstat = reinterpret_cast<float2*>(w + lay.rowstat);
  a.diag_part = reinterpret_cast<float2*>(w + lay.diag_part);
  a.rk_hist = reinterpret_cast<uint32_t*>(w + lay.rk_hist);
  a.rk_state = reinterpret_cast<uint32_t*>(w + lay.rk_state);
  const bool direct = ch.c1 <= 4;
  a.stat = direct ? a.part : a.rowstat;
  a.cs = direct ? (int32_t)ch.c1 : 1;

  const bool xf = (tu != nullptr) || (p->temperature != 1.0f) || (p->top_k > 0);
  hipError_t e = csd::launch_diagnostics(a, p->dtype, xf, local, static_cast<hipStream_t>(stream), false);
  return e == hipSuccess ? COOL_SD_OK : COOL_SD_ELAUNCH;
}

// cool_sd_verify_diagnostics on rows of one chunk without top-k: one pass over the logits leaves
// the verify call's statistics and alpha, beta; the per-sequence kernel follows.
int run_verify_diag(const cool_sd_params* p, const void* t, const void* tu, const void* d, const void* du,
                    const int32_t* tokens, const float* omega, const float* u_acc, const float* u_res,
                    int32_t* accept_len, int32_t* next_token, float* p_tok, float* q_tok, float* f,
                    float* resid_mass, float* alpha, float* beta, void* ws, size_t ws_bytes, void* stream) {
  const int64_t L = p->L;
  const int64_t rows_t = int64_t(p->B) * (L + p->has_bonus), rows_d = int64_t(p->B) * L;
  const Layout lay = make_layout(p->B, rows_t + rows_d, 1, 1);
  if (!ws || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0 || ws_bytes < lay.total) return COOL_SD_EWORKSPACE;
  const int kE = (p->dtype == COOL_SD_BF16) ? 8 : 4;
  bool aligned = (p->V % kE == 0) && is_aligned16(t) && is_aligned16(d) && (p->t_stride_b % kE == 0) &&
                 (p->t_stride_l % kE == 0) && (p->d_stride_b % kE == 0) && (p->d_stride_l % kE == 0);
  if (tu) aligned = aligned && is_aligned16(tu) && is_aligned16(du);

  char* w = static_cast<char*>(ws);
  csd::KArgs a{};
  a.t = t; a.tu = tu; a.d = d; a.du = du;
  a.tokens = tokens; a.omega = omega; a.u_acc = u_acc; a.u_res = u_res;
  a.accept_len = accept_len; a.next_token = next_token;
  a.p_tok = p_tok; a.q_tok = q_tok; a.f = f; a.resid_mass = resid_mass;
  a.alpha = alpha; a.beta = beta;
  a.t_sb = p->t_stride_b; a.t_sl = p->t_stride_l; a.d_sb = p->d_stride_b; a.d_sl = p->d_stride_l;
  a.om_sb = p->omega_stride_b;
  a.B = p->B; a.L = (int32_t)L; a.V = p->V; a.has_bonus = p->has_bonus;
  a.top_k = 0; a.resample_mode = p->resample_mode;
  a.exact_draw = (p->flags & COOL_SD_FLAG_EXACT_DRAW) ? 1 : 0;
  a.aligned = aligned ? 1 : 0;
  a.nchunks = 1;                                  // one sampling chunk, one diagnostics chunk
  const int kT = (p->dtype == COOL_SD_BF16) ? 8 : 16;
  a.nt2 = kT;
  a.cfg_scale = p->cfg_scale;
  a.inv_T = 1.0f / p->temperature;
  a.rows_t = (int32_t)rows_t; a.rows_d = (int32_t)rows_d;
  a.nt1 = kT; a.chunk1 = csd::kChunk; a.c1 = 1;   // one statistics pair per row
  a.chunk_R = reinterpret_cast<float*>(w + lay.chunk_R);
  a.seq_stat = reinterpret_cast<float4*>(w + lay.seq_stat);
  a.ticket = reinterpret_cast<int32_t*>(w + lay.ticket);
  a.thr = reinterpret_cast<float*>(w + lay.thr);
  a.tok_logit = reinterpret_cast<float*>(w + lay.tok_logit);
  a.part = reinterpret_cast<float2*>(w + lay.part);
  a.rowstat = reinterpret_cast<float2*>(w + lay.rowstat);
  a.stat = a.part;
  a.cs = 1;
  const bool xf = (tu != nullptr) || (p->temperature != 1.0f);
  hipError_t e = csd::launch_verify_diagnostics(a, p->dtype, xf, static_cast<hipStream_t>(stream));
  if (e == hipSuccess && (call_flags(p) & COOL_SD_FLAG_CHECK_TOKENS)) e = csd::launch_check_tokens(a, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? COOL_SD_OK : COOL_SD_ELAUNCH;
}

}  // namespace
}  // namespace csd_api
