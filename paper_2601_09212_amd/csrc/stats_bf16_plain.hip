// Statistics pass, bf16 logits as they are.
#include "stats_launch.h"

namespace csd {

hipError_t launch_statistics_bf16_plain(const KArgs& a, hipStream_t stream) {
  return a.aligned ? launch_stats_any<kDtBF16, false, true>(a, stream) : launch_stats_any<kDtBF16, false, false>(a, stream);
}

}  // namespace csd
