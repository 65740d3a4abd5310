// C ABI of the Cool-SD verify-and-resample library: argument validation, workspace layout,
// the host-side relaxation schedule, and kernel dispatch.  See include/cool_sd.h.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "cool_sd.h"
#include "device_utils.h"
#include "kernels.h"

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layout {
  size_t seq_stat, chunk_R, thr, tok_logit, rowstat, part, diag_part, lan, rk_hist, rk_state, total;
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
  if ((p->flags & ~COOL_SD_FLAG_EARLY_EXIT) != 0) return false;
  const int64_t L = for_resample ? 1 : p->L;
  const int64_t rows = for_resample ? p->B : int64_t(p->B) * (L + p->has_bonus);
  if (2 * rows * ((int64_t(p->V) + 4095) / 4096) > 0x7fffffffLL) return false;   // grid size
  return true;
}

// benchmark instrumentation (see cool_sd_profile_enable)
bool g_profile = false;
bool g_stats_only = false;   // benchmark mode 2: enqueue the statistics kernel alone
bool g_profile_valid = false;
hipEvent_t g_ev[3] = {nullptr, nullptr, nullptr};

inline bool is_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int run(const cool_sd_params* p, bool resample_only,
        const void* t, const void* tu, const void* d, const void* du,
        const int32_t* tokens, const float* omega, const float* u_acc, const float* u_res,
        int32_t* accept_len, int32_t* next_token, float* p_tok, float* q_tok, float* f,
        float* resid_mass, void* ws, size_t ws_bytes, void* stream, const LanternArgs* lan = nullptr,
        float* alpha = nullptr, float* beta = nullptr) {
  const int64_t L = resample_only ? 1 : p->L;
  const int hb = resample_only ? 0 : p->has_bonus;
  const int64_t rows = resample_only ? p->B : int64_t(p->B) * (L + hb);
  const int64_t rows_t = rows, rows_d = d ? int64_t(p->B) * L : 0;
  const Chunking ch = pick_chunking(p, rows_t + rows_d);
  const int64_t C = ch.c2;
  const bool radix = p->top_k > 0 && p->V > 4 * csd::kChunk;
  // with alpha / beta the diagnostics pass follows on the statistics this call leaves (8192-logit chunks)
  const int64_t pairs = alpha ? int64_t(p->B) * L : 0, CD = alpha ? (int64_t(p->V) + 8191) / 8192 : 0;
  const Layout lay = make_layout(p->B, rows_t + rows_d, ch.c1, C, pairs, CD, lan ? int64_t(p->B) * L : 0,
                                 radix ? rows_t + rows_d : 0);
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
  a.stats_only = g_stats_only ? 1 : 0;
  a.early_exit = (!resample_only && !lan && aligned && (p->flags & COOL_SD_FLAG_EARLY_EXIT) && p->top_k == 0 &&
                  p->V <= csd::kChunk && p->L <= 1024) ? 1 : 0;
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
  a.cfg_scale = p->cfg_scale;
  a.inv_T = 1.0f / p->temperature;
  a.rows_t = (int32_t)rows_t; a.rows_d = (int32_t)rows_d;
  a.nt1 = ch.nt1; a.chunk1 = ch.chunk1; a.c1 = (int32_t)ch.c1;
  a.chunk_R = reinterpret_cast<float*>(w + lay.chunk_R);
  a.seq_stat = reinterpret_cast<float4*>(w + lay.seq_stat);
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
  hipError_t e = csd::launch_verify(a, p->dtype, xf, static_cast<hipStream_t>(stream), g_profile ? g_ev : nullptr);
  g_profile_valid = g_profile && e == hipSuccess;
  if (e == hipSuccess && alpha && !g_stats_only) {
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
  a.thr = reinterpret_cast<float*>(w + lay.thr);
  a.tok_logit = reinterpret_cast<float*>(w + lay.tok_logit);
  a.part = reinterpret_cast<float2*>(w + lay.part);
  a.rowstat = reinterpret_cast<float2*>(w + lay.rowstat);
  a.stat = a.part;
  a.cs = 1;
  const bool xf = (tu != nullptr) || (p->temperature != 1.0f);
  hipError_t e = csd::launch_verify_diagnostics(a, p->dtype, xf, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? COOL_SD_OK : COOL_SD_ELAUNCH;
}

}  // namespace

extern "C" {

int cool_sd_schedule(int32_t kind, int32_t L, float delta, float param, float* omega_out) {
  if (L < 1 || L > 4096 || !omega_out || !(delta >= 0.f) || !isfinite(delta)) return COOL_SD_EINVAL;
  if (kind == COOL_SD_SCHED_UNIFORM) {
    for (int i = 0; i < L; ++i) omega_out[i] = delta;
    return COOL_SD_OK;
  }
  if (kind == COOL_SD_SCHED_EXP) {
    // omega_i = delta exp(-nu i - mu) with sum_i exp(-nu i - mu) = L, i.e. the weights
    // exp(-nu i) rescaled to sum to L (Eq. sdar).  Anchored at i = 1 to stay in range.
    const double nu = param;
    if (!(nu > 0.0) || !isfinite(nu)) return COOL_SD_EINVAL;
    double z = 0.0;
    for (int i = L; i >= 1; --i) z += exp(-nu * double(i - 1));
    for (int i = 1; i <= L; ++i)
      omega_out[i - 1] = float(double(delta) * double(L) * exp(-nu * double(i - 1)) / z);
    return COOL_SD_OK;
  }
  if (kind == COOL_SD_SCHED_LINEAR) {
    // omega_i proportional to (ell - i), rescaled to sum to delta L; the common factor
    // 1/(ell (ell+1)) of the paper's weights cancels (App., schedule ablation).
    const double ell = param;
    if (!(ell >= double(L)) || !isfinite(ell)) return COOL_SD_EINVAL;
    const double z = double(L) * ell - 0.5 * double(L) * double(L + 1);
    if (!(z > 0.0)) return COOL_SD_EINVAL;
    for (int i = 1; i <= L; ++i) omega_out[i - 1] = float(double(delta) * double(L) * (ell - double(i)) / z);
    return COOL_SD_OK;
  }
  return COOL_SD_EINVAL;
}

size_t cool_sd_workspace_bytes(const cool_sd_params* p) {
  if (!params_ok(p, false, true) && !params_ok(p, true)) return 0;
  const bool full = params_ok(p, false, true);
  const int64_t L = full ? p->L : 1;
  const int64_t rows = full ? int64_t(p->B) * (2 * L + p->has_bonus) : 2 * int64_t(p->B);
  // sized for the finest chunking so that the answer does not depend on optional inputs
  const int64_t c1_max = (int64_t(p->V) + 4095) / 4096;
  const int64_t pairs = full ? int64_t(p->B) * L : 0;       // cool_sd_diagnostics: chunks of 8192 logits
  const bool radix = p->top_k > 0 && p->V > 4 * csd::kChunk;
  return make_layout(p->B, rows, c1_max, c1_max, pairs, (int64_t(p->V) + 8191) / 8192, pairs, radix ? rows : 0).total;
}

int cool_sd_workspace_init(void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) % kAlign) != 0) return COOL_SD_EWORKSPACE;
  hipError_t e = csd::launch_zero(static_cast<uint32_t*>(workspace_dev), workspace_bytes / 4,
                                  static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? COOL_SD_OK : COOL_SD_ELAUNCH;
}

int cool_sd_verify(const cool_sd_params* p, const void* target_dev, const void* target_uncond_dev,
                   const void* draft_dev, const void* draft_uncond_dev, const int32_t* draft_tokens_dev,
                   const float* omega_dev, const float* u_accept_dev, const float* u_resample_dev,
                   int32_t* accept_len_dev, int32_t* next_token_dev, float* p_tok_dev, float* q_tok_dev,
                   float* f_dev, float* resid_mass_dev, void* workspace_dev, size_t workspace_bytes,
                   void* hip_stream) {
  if (!params_ok(p, false)) return COOL_SD_EINVAL;
  if (!target_dev || !draft_dev || !draft_tokens_dev || !omega_dev || !u_accept_dev || !u_resample_dev ||
      !accept_len_dev || !next_token_dev)
    return COOL_SD_EINVAL;
  if ((target_uncond_dev == nullptr) != (draft_uncond_dev == nullptr)) return COOL_SD_EINVAL;
  return run(p, false, target_dev, target_uncond_dev, draft_dev, draft_uncond_dev, draft_tokens_dev, omega_dev,
             u_accept_dev, u_resample_dev, accept_len_dev, next_token_dev, p_tok_dev, q_tok_dev, f_dev,
             resid_mass_dev, workspace_dev, workspace_bytes, hip_stream);
}

int cool_sd_verify_lantern(const cool_sd_params* p, const void* target_dev, const void* target_uncond_dev,
                           const void* draft_dev, const void* draft_uncond_dev, const int32_t* draft_tokens_dev,
                           const int32_t* neighbors_dev, int32_t k, float lambda, const float* u_accept_dev,
                           const float* u_resample_dev, int32_t* accept_len_dev, int32_t* next_token_dev,
                           float* p_tok_dev, float* q_tok_dev, float* f_dev, float* resid_mass_dev, float* p_agg_dev,
                           int32_t* count_dev, void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!params_ok(p, false, true)) return COOL_SD_EINVAL;
  if (!target_dev || !draft_dev || !draft_tokens_dev || !u_accept_dev || !u_resample_dev || !accept_len_dev ||
      !next_token_dev)
    return COOL_SD_EINVAL;
  if ((target_uncond_dev == nullptr) != (draft_uncond_dev == nullptr)) return COOL_SD_EINVAL;
  if (k < 1 || k > 65536 || !neighbors_dev || !(lambda >= 0.f) || !isfinite(lambda)) return COOL_SD_EINVAL;
  const LanternArgs lan{neighbors_dev, k, lambda, p_agg_dev, count_dev};
  return run(p, false, target_dev, target_uncond_dev, draft_dev, draft_uncond_dev, draft_tokens_dev, nullptr,
             u_accept_dev, u_resample_dev, accept_len_dev, next_token_dev, p_tok_dev, q_tok_dev, f_dev,
             resid_mass_dev, workspace_dev, workspace_bytes, hip_stream, &lan);
}

int cool_sd_resample(const cool_sd_params* p, const void* target_rows_dev, const void* target_uncond_rows_dev,
                     const void* draft_rows_dev, const void* draft_uncond_rows_dev, const float* omega_rows_dev,
                     const float* u_dev, int32_t* token_dev, float* resid_mass_dev, void* workspace_dev,
                     size_t workspace_bytes, void* hip_stream) {
  if (!params_ok(p, true)) return COOL_SD_EINVAL;
  if (!target_rows_dev || !u_dev || !token_dev) return COOL_SD_EINVAL;
  if (draft_rows_dev && !omega_rows_dev) return COOL_SD_EINVAL;
  if (!draft_rows_dev && draft_uncond_rows_dev) return COOL_SD_EINVAL;
  if (draft_rows_dev && ((target_uncond_rows_dev == nullptr) != (draft_uncond_rows_dev == nullptr)))
    return COOL_SD_EINVAL;
  return run(p, true, target_rows_dev, target_uncond_rows_dev, draft_rows_dev, draft_uncond_rows_dev, nullptr,
             omega_rows_dev, nullptr, u_dev, nullptr, token_dev, nullptr, nullptr, nullptr, resid_mass_dev,
             workspace_dev, workspace_bytes, hip_stream);
}

int cool_sd_diagnostics(const cool_sd_params* p, const void* target_dev, const void* target_uncond_dev,
                        const void* draft_dev, const void* draft_uncond_dev, const float* omega_dev,
                        float* alpha_dev, float* beta_dev, void* workspace_dev, size_t workspace_bytes,
                        void* hip_stream) {
  if (!params_ok(p, false)) return COOL_SD_EINVAL;
  if (!target_dev || !draft_dev || !omega_dev || !alpha_dev || !beta_dev) return COOL_SD_EINVAL;
  if ((target_uncond_dev == nullptr) != (draft_uncond_dev == nullptr)) return COOL_SD_EINVAL;
  return run_diag(p, target_dev, target_uncond_dev, draft_dev, draft_uncond_dev, omega_dev, alpha_dev, beta_dev,
                  workspace_dev, workspace_bytes, hip_stream);
}

int cool_sd_verify_diagnostics(const cool_sd_params* p, const void* target_dev, const void* target_uncond_dev,
                               const void* draft_dev, const void* draft_uncond_dev, const int32_t* draft_tokens_dev,
                               const float* omega_dev, const float* u_accept_dev, const float* u_resample_dev,
                               int32_t* accept_len_dev, int32_t* next_token_dev, float* p_tok_dev, float* q_tok_dev,
                               float* f_dev, float* resid_mass_dev, float* alpha_dev, float* beta_dev,
                               void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!params_ok(p, false)) return COOL_SD_EINVAL;
  if (!target_dev || !draft_dev || !draft_tokens_dev || !omega_dev || !u_accept_dev || !u_resample_dev ||
      !accept_len_dev || !next_token_dev || !alpha_dev || !beta_dev)
    return COOL_SD_EINVAL;
  if ((target_uncond_dev == nullptr) != (draft_uncond_dev == nullptr)) return COOL_SD_EINVAL;
  if (p->top_k == 0 && p->V <= csd::kChunk && !g_profile && !g_stats_only)
    return run_verify_diag(p, target_dev, target_uncond_dev, draft_dev, draft_uncond_dev, draft_tokens_dev, omega_dev,
                           u_accept_dev, u_resample_dev, accept_len_dev, next_token_dev, p_tok_dev, q_tok_dev, f_dev,
                           resid_mass_dev, alpha_dev, beta_dev, workspace_dev, workspace_bytes, hip_stream);
  // top-k or rows of several chunks: the verify call, then the diagnostics pass on the row
  // statistics and thresholds it left (the early-exit flag is not honoured here, the diagnostics
  // need every row anyway)
  cool_sd_params q = *p;
  q.flags = 0;
  return run(&q, false, target_dev, target_uncond_dev, draft_dev, draft_uncond_dev, draft_tokens_dev, omega_dev,
             u_accept_dev, u_resample_dev, accept_len_dev, next_token_dev, p_tok_dev, q_tok_dev, f_dev,
             resid_mass_dev, workspace_dev, workspace_bytes, hip_stream, nullptr, alpha_dev, beta_dev);
}

int cool_sd_profile_enable(int enable) {
  if (enable < 0 || enable > 2) return COOL_SD_EINVAL;
  if (enable == 1 && !g_ev[0]) {
    for (int i = 0; i < 3; ++i)
      if (hipEventCreate(&g_ev[i]) != hipSuccess) return COOL_SD_ELAUNCH;
  }
  g_profile = enable == 1;
  g_stats_only = enable == 2;
  g_profile_valid = false;
  return COOL_SD_OK;
}

int cool_sd_profile_read(float* stats_kernel_ms, float* call_ms) {
  if (!g_profile_valid || !stats_kernel_ms || !call_ms) return COOL_SD_EINVAL;
  if (hipEventSynchronize(g_ev[2]) != hipSuccess) return COOL_SD_ELAUNCH;
  if (hipEventElapsedTime(stats_kernel_ms, g_ev[0], g_ev[1]) != hipSuccess) return COOL_SD_ELAUNCH;
  if (hipEventElapsedTime(call_ms, g_ev[0], g_ev[2]) != hipSuccess) return COOL_SD_ELAUNCH;
  return COOL_SD_OK;
}

int cool_sd_profile_read_probe(const void* a_dev, size_t a_bytes, const void* b_dev, size_t b_bytes,
                               void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!a_dev || a_bytes == 0 || (a_bytes % 16) != 0 || (b_bytes % 16) != 0 || !is_aligned16(a_dev) ||
      (b_bytes != 0 && (!b_dev || !is_aligned16(b_dev))))
    return COOL_SD_EINVAL;
  const size_t na = a_bytes / 16, nb = b_bytes / 16;
  const size_t groups = (na + csd::kProbeVecsPerGroup - 1) / csd::kProbeVecsPerGroup +
                        (nb + csd::kProbeVecsPerGroup - 1) / csd::kProbeVecsPerGroup;
  if (groups > 0x7fffffffULL) return COOL_SD_EINVAL;
  if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) % 4) != 0 || workspace_bytes < groups * 4)
    return COOL_SD_EWORKSPACE;
  hipError_t e = csd::launch_read_probe(static_cast<const uint4*>(a_dev), na, static_cast<const uint4*>(b_dev), nb,
                                        static_cast<uint32_t*>(workspace_dev), static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? COOL_SD_OK : COOL_SD_ELAUNCH;
}

const char* cool_sd_strerror(int code) {
  switch (code) {
    case COOL_SD_OK: return "ok";
    case COOL_SD_EINVAL: return "invalid argument";
    case COOL_SD_EWORKSPACE: return "workspace missing, misaligned or too small";
    case COOL_SD_ELAUNCH: return "HIP launch failed";
    case COOL_SD_EUNSUPPORTED: return "request not implemented by the kernels";
    default: return "unknown status";
  }
}

}  // extern "C"
