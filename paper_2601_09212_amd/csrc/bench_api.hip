// Entry points of the benchmark library libcool_sd_bench.so (include/cool_sd_bench.h): the
// statistics pass of a verify call on its own, and a plain streaming read as a yardstick.  Built
// from the same kernels as libcool_sd.so; the product library exports none of this.
#include "api_core.h"
#include "cool_sd_bench.h"

using namespace csd_api;

extern "C" {

int cool_sd_bench_row_stats(const cool_sd_params* p, const void* target_dev, const void* target_uncond_dev,
                            const void* draft_dev, const void* draft_uncond_dev, const int32_t* draft_tokens_dev,
                            void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
  if (!params_ok(p, false)) return COOL_SD_EINVAL;
  if (!target_dev || !draft_dev || !draft_tokens_dev) return COOL_SD_EINVAL;
  if ((target_uncond_dev == nullptr) != (draft_uncond_dev == nullptr)) return COOL_SD_EINVAL;
  cool_sd_params q = *p;
  q.flags = 0;
  return run(&q, false, target_dev, target_uncond_dev, draft_dev, draft_uncond_dev, draft_tokens_dev, nullptr, nullptr,
             nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, workspace_dev, workspace_bytes, hip_stream,
             nullptr, nullptr, nullptr, /*stats_only=*/true);
}

int cool_sd_bench_read_probe(const void* a_dev, size_t a_bytes, const void* b_dev, size_t b_bytes,
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

}  // extern "C"
