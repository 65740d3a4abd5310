// Statistics pass, f32 logits as they are.
#include "stats_launch.h"

namespace csd {

hipError_t launch_statistics_f32_plain(const KArgs& a, hipStream_t stream) {
  return a.aligned ? launch_stats_any<kDtF32, false, true>(a, stream) : launch_stats_any<kDtF32, false, false>(a, stream);
}

}  // namespace csd
