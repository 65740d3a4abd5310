// Statistics pass, bf16 logits with a logit transform (guidance / temperature / top-k).
#include "stats_launch.h"

namespace csd {

hipError_t launch_statistics_bf16_xf(const KArgs& a, hipStream_t stream) {
  return a.aligned ? launch_stats_any<kDtBF16, true, true>(a, stream) : launch_stats_any<kDtBF16, true, false>(a, stream);
}

hipError_t launch_resample_topk_bf16(const KArgs& a, hipStream_t stream) {
  return a.aligned ? launch_resample_topk_typed<kDtBF16, kAligned>(a, stream) : launch_resample_topk_typed<kDtBF16, kUnaligned>(a, stream);
}

}  // namespace csd
