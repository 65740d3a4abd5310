// C ABI of the Cool-SD verify-and-resample library: the entry points of include/cool_sd.h.
#include <atomic>

#include "api_core.h"

using namespace csd_api;

namespace {

// cool_sd_verify_noalloc: the call's workspace lives in this array instead of caller memory.  Every
// GPU the library runs on holds its own copy at its own address until the process ends; the name
// below is only the host-side stand-in of the symbol, so the device address is looked up once per
// device (hipGetSymbolAddress, with that device current) and kept.  The per-device pointers are
// the only state of the library: written once each, to a value that never changes.
constexpr size_t kStaticWorkspaceBytes = size_t(COOL_SD_NOALLOC_WORKSPACE_BYTES);
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];
constexpr int kMaxDevices = 64;
std::atomic<void*> scratch_ptr[kMaxDevices];

int static_workspace(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return COOL_SD_ELAUNCH;
  void* ptr = scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return COOL_SD_ELAUNCH;
    scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return COOL_SD_OK;
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

int cool_sd_verify_noalloc(const cool_sd_params* p, const void* target_dev, const void* target_uncond_dev,
                           const void* draft_dev, const void* draft_uncond_dev, const int32_t* draft_tokens_dev,
                           const float* omega_dev, const float* u_accept_dev, const float* u_resample_dev,
                           int32_t* accept_len_dev, int32_t* next_token_dev, float* p_tok_dev, float* q_tok_dev,
                           float* f_dev, float* resid_mass_dev, void* hip_stream) {
  if (!params_ok(p, false)) return COOL_SD_EINVAL;
  if (!target_dev || !draft_dev || !draft_tokens_dev || !omega_dev || !u_accept_dev || !u_resample_dev ||
      !accept_len_dev || !next_token_dev)
    return COOL_SD_EINVAL;
  if ((target_uncond_dev == nullptr) != (draft_uncond_dev == nullptr)) return COOL_SD_EINVAL;
  // the size is known from the params alone: refuse before anything touches the device
  if (plan_call(p, false, true, false, false).lay.total > kStaticWorkspaceBytes) return COOL_SD_ETOOLARGE;
  void* ws = nullptr;
  const int rc = static_workspace(&ws);
  if (rc != COOL_SD_OK) return rc;
  return run(p, false, target_dev, target_uncond_dev, draft_dev, draft_uncond_dev, draft_tokens_dev, omega_dev,
             u_accept_dev, u_resample_dev, accept_len_dev, next_token_dev, p_tok_dev, q_tok_dev, f_dev,
             resid_mass_dev, ws, kStaticWorkspaceBytes, hip_stream);
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
  if (p->top_k == 0 && p->V <= csd::kChunk)
    return run_verify_diag(p, target_dev, target_uncond_dev, draft_dev, draft_uncond_dev, draft_tokens_dev, omega_dev,
                           u_accept_dev, u_resample_dev, accept_len_dev, next_token_dev, p_tok_dev, q_tok_dev, f_dev,
                           resid_mass_dev, alpha_dev, beta_dev, workspace_dev, workspace_bytes, hip_stream);
  // top-k or rows of several chunks: the verify call, then the diagnostics pass on the row
  // statistics and thresholds it left (the early-exit flag is not honoured here, the diagnostics
  // need every row anyway)
  cool_sd_params q = *p;
  q.flags &= ~COOL_SD_FLAG_EARLY_EXIT;
  return run(&q, false, target_dev, target_uncond_dev, draft_dev, draft_uncond_dev, draft_tokens_dev, omega_dev,
             u_accept_dev, u_resample_dev, accept_len_dev, next_token_dev, p_tok_dev, q_tok_dev, f_dev,
             resid_mass_dev, workspace_dev, workspace_bytes, hip_stream, nullptr, alpha_dev, beta_dev);
}

int cool_sd_early_exit_form(const cool_sd_params* p, int rows_aligned) {
  if (!params_ok(p, /*for_resample=*/false)) return COOL_SD_EINVAL;
  const int kE = (p->dtype == COOL_SD_BF16) ? 8 : 4;
  return early_exit_form(p, rows_aligned != 0 && p->V % kE == 0);
}

const char* cool_sd_strerror(int code) {
  switch (code) {
    case COOL_SD_OK: return "ok";
    case COOL_SD_EINVAL: return "invalid argument";
    case COOL_SD_EWORKSPACE: return "workspace missing, misaligned or too small";
    case COOL_SD_ELAUNCH: return "HIP launch failed";
    case COOL_SD_EUNSUPPORTED: return "request not implemented by the kernels";
    case COOL_SD_ETOOLARGE: return "shape needs more workspace than the library's static array holds";
    default: return "unknown status";
  }
}

}  // extern "C"
