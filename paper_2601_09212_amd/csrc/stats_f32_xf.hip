// Statistics pass, f32 logits with a logit transform (guidance / temperature / top-k).
#include "stats_launch.h"

namespace csd {

hipError_t launch_statistics_f32_xf(const KArgs& a, hipStream_t stream) {
  return a.aligned ? launch_stats_any<kDtF32, true, true>(a, stream) : launch_stats_any<kDtF32, true, false>(a, stream);
}

hipError_t launch_resample_topk_f32(const KArgs& a, hipStream_t stream) {
  return a.aligned ? launch_resample_topk_typed<kDtF32, kAligned>(a, stream) : launch_resample_topk_typed<kDtF32, kUnaligned>(a, stream);
}

}  // namespace csd
